#!/usr/bin/env python3
"""Benchmark of the generation hot path on one MI355X.

A "step" is one pass of the whole hot path: fg_generate over one block of synthetic prompts
(prefill of all GPU batches, then n-1 decode steps), inputs already resident in HBM.  The default
workload is the one the headline metric is quoted on: OPT-175B shape, 4-bit group-wise weights and
KV cache, block 4 x 36 sequences, prompt 512, 32 generated tokens (Section 6 workload of the paper).

Prints ONE JSON line with generated tokens/s (paper's definition: bls*n / (prefill + decode time)),
the per-kernel-class rooflines measured live with HIP events on the launch stream, the decode-phase
HBM fraction, and the CPU oracle timed on a bounded slice of the same workload.

One pass of the headline workload takes about 25 s, so --steps and --warmup are UPPER BOUNDS under a
wall-clock budget (--budget-s, counted from process start): after the first pass has been timed, the
number of passes that still fit is planned (plan_passes), and the line reports the counts actually
run.  The timed passes carry HIP events only on the few long prefill kernels (a pair of events costs
microseconds per launch, which a decode step of a thousand short launches would feel); one extra,
untimed pass with events on every launch gives the per-kernel-class table.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

T_PROCESS_START = time.perf_counter()
ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK = 8.0e12          # bytes/s, MI355X HBM3E
MFMA_F16_PEAK = 2.5e15     # flop/s, dense FP16 MFMA

WORKLOADS = {
    # name: (shape name, quantized weights, quantized kv, num_gpu_batches, gpu_batch_size, s, n)
    "opt175b_q4": ("OPT_175B", True, True, 4, 36, 512, 32),
    # schedule ablation (Section 4.2): ONE GPU batch of the 175B block per pass over the layers, i.e. what
    # the row-by-row order costs: every 36 sequences stream all weights again
    "opt175b_q4_1x36": ("OPT_175B", True, True, 1, 36, 512, 32),
    # other prompt/generation lengths of the paper's evaluation (Section 6 and its appendix tables)
    "opt175b_q4_1024_32": ("OPT_175B", True, True, 4, 20, 1024, 32),
    "opt175b_q4_128_128": ("OPT_175B", True, True, 4, 36, 128, 128),
    "opt175b_q4_512_8": ("OPT_175B", True, True, 4, 36, 512, 8),
    # the 4.5-bit cache variant: FP16 {min, scale} pairs (10 % fewer KV bytes per step)
    "opt175b_q4_h16kv": ("OPT_175B", True, "h16", 4, 36, 512, 32),
    # ... and with the weights' pairs in FP16 as well: 4.5 bits per stored element everywhere
    "opt175b_q4_h16": ("OPT_175B", "h16", "h16", 4, 36, 512, 32),
    "kv_stress_175b_layer_h16kv": ("OPT_175B", True, "h16", 1, 512, 2048, 64),
    # the appendix's diagonal block schedule over paged caches (run_diagonal): the same 144 sequences
    # admitted four at a time; and the 128+128 setting, where the staggered lengths save cache memory
    "opt175b_q4_diagonal": ("OPT_175B", True, True, 36, 4, 512, 32),
    "opt175b_q4_128_128_diagonal": ("OPT_175B", True, True, 36, 4, 128, 128),
    "opt30b_q4": ("OPT_30B", True, True, 8, 32, 512, 32),
    "opt6.7b_f16": ("OPT_6_7B", False, False, 4, 32, 512, 32),
    "opt125m_layer_q4": ("OPT_125M_LAYER", True, True, 1, 4, 32, 9),
    # KV-bound decode stress: ONE OPT-175B-shaped layer, batch 512, 2048 cached rows, 64 decode steps
    # (handled by run_kv_stress: the cache is filled synthetically, there is no prefill)
    "kv_stress_175b_layer": ("OPT_175B", True, True, 1, 512, 2048, 64),
}


# kernel classes that are few, long launches in a generation pass: timing them inside the timed region
# costs nothing measurable (about 2000 event pairs per pass against 25 s)
CHEAP_TO_TIME = ("gemm_large_m", "attn_prefill")


def plan_passes(steps, warmup, pass_s, avail_s):
    """How many passes to run when ONE pass has already been run and took pass_s seconds and avail_s
    seconds are left for further warm-up and timed passes.  steps / warmup are the requested counts,
    taken as upper bounds.  The pass already run is the first warm-up pass if warmup >= 1, otherwise the
    first timed pass.  Timed passes have priority over further warm-up passes; at least one pass is
    timed whatever the budget says.  Returns (warmup passes in total, timed passes in total)."""
    steps = max(1, int(steps))
    warmup = max(0, int(warmup))
    fit = int(avail_s // pass_s) if pass_s > 0 and avail_s > 0 else 0
    if warmup == 0:
        return 0, 1 + min(steps - 1, fit)
    k = min(steps, max(1, fit))
    w = 1 + min(warmup - 1, max(0, fit - k))
    return w, k


def bpe(q):
    """Stored bytes per element: FP16, 4-bit with binary32 pairs, or ("h16") 4-bit with FP16 pairs."""
    return 0.5625 if q == "h16" else (0.625 if q else 2.0)


def build_model(sh, wq, seed, torch, B, embeddings=True):
    """Random-init weights ~N(0, 0.02) generated and quantized on the device, one layer at a time."""
    g = torch.Generator(device="cuda")
    layers = []
    ones = torch.ones(sh.h1, dtype=torch.float16, device="cuda")
    zeros = torch.zeros(sh.h1, dtype=torch.float16, device="cuda")

    def mat(rows, cols, j, tid):
        g.manual_seed(seed * 1000003 + j * 16 + tid)
        w = torch.empty((rows, cols), dtype=torch.float16, device="cuda")
        w.normal_(0.0, 0.02, generator=g)
        # 4-bit matrices go into the tiled streaming layout (same bytes, repacked once at load time)
        m = B.Mat.from_f16(w, bool(wq), tiled=bool(wq), meta_f16=wq == "h16")
        return m

    for j in range(sh.l):
        layers.append(B.LayerWeights(mat(3 * sh.h1, sh.h1, j, 0), mat(sh.h1, sh.h1, j, 1), mat(sh.h2, sh.h1, j, 2),
                                     mat(sh.h1, sh.h2, j, 3), ones, zeros, ones, zeros))
    if not embeddings:
        return layers, None, None, ones, zeros
    g.manual_seed(seed * 1000003 + 999983)
    emb = torch.empty((sh.vocab, sh.h1), dtype=torch.float16, device="cuda").normal_(0.0, 0.02, generator=g)
    pos = torch.empty((sh.max_pos, sh.h1), dtype=torch.float16, device="cuda").normal_(0.0, 0.02, generator=g)
    return layers, emb, pos, ones, zeros


def cpu_baseline(sh, wq, kvq, s, n, bls, budget_s=25.0):
    """The oracle as it stands (numpy, float64; its matrix products run on numpy's BLAS threads), on
    the host cores, on a bounded slice of the workload at the real widths: ONE layer, the decode step
    of 4 sequences at the mean cache length and the prefill of one sequence, each projection cut to a
    slab of rows of its weight matrix and the attention to as many heads as fit the time budget; the
    pieces are scaled to the full matrices / all heads, then to l layers, s + n - 1 positions and the
    whole block, giving the same quantity as the headline: generated tokens per second of the block,
    bls * n / (prefill + decode).  Reported, not a target."""
    import numpy as np
    from oracle import fg_oracle as O
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        threads = os.cpu_count() or 1
    t_begin = time.perf_counter()
    b, slab = 4, 3072
    rows = s + n // 2
    h1, h2, nh, dh = sh.h1, sh.h2, sh.nh, sh.dh
    rng = np.random.default_rng(0)
    f16 = lambda shape, std: (rng.standard_normal(shape, dtype=np.float32) * np.float32(std)).astype(np.float16)
    slabs = {"wqkv": (3 * h1, h1), "wo": (h1, h1), "w1": (h2, h1), "w2": (h1, h2)}
    mats = {k: O.Mat.from_f16(f16((min(slab, r), c), 0.02), bool(wq), wq == "h16") for k, (r, c) in slabs.items()}
    ones, zeros = np.ones(h1, np.float16), np.zeros(h1, np.float16)

    def linears(x, a):
        """all four projections on x [m, h1] / a [m, h2], seconds scaled to the full matrices"""
        t = 0.0
        for k, (r, c) in slabs.items():
            xin = a if k == "w2" else x
            t0 = time.perf_counter()
            O.round_f16(O.linear(xin, mats[k], None))
            t += (time.perf_counter() - t0) * (r / min(slab, r))
        return t

    def layernorms(x):
        t0 = time.perf_counter()
        O.round_f16(O.layernorm(x.astype(np.float64), ones, zeros, 1e-5))
        return 2 * (time.perf_counter() - t0)

    # ---- decode step of one layer, b sequences
    kv = O.KVCache.empty(b, nh, rows + 1, dh, bool(kvq), kvq == "h16")
    kv.store(0, 0, f16((b, rows, h1), 1.0), f16((b, rows, h1), 1.0))
    x, a = f16((b, h1), 1.0), f16((b, h2), 1.0)
    t_dec = layernorms(x) + linears(x, a)
    t0 = time.perf_counter()
    kv.store(0, rows, f16((b, 1, h1), 1.0), f16((b, 1, h1), 1.0))
    q = x.astype(np.float64).reshape(b, nh, dh)
    heads = 0
    for bi in range(b):
        for h in range(nh):
            kh, vh = kv.load(bi, h, rows + 1)
            O.attn_decode(q[bi, h], kh, vh)
            heads += 1
        if time.perf_counter() - t0 > budget_s * 0.3:
            break
    t_dec += (time.perf_counter() - t0) * (b * nh / max(heads, 1))
    t_dec_seq = t_dec / b                                  # seconds per sequence, layer and decode step
    # ---- prefill of one layer, one sequence of s positions
    xs, as_ = f16((s, h1), 1.0), f16((s, h2), 1.0)
    t_pre = layernorms(xs) + linears(xs, as_)
    qkv = f16((s, 3, nh, dh), 1.0).astype(np.float64)
    t0 = time.perf_counter()
    heads = 0
    for h in range(nh):
        O.attn_prefill(qkv[:, 0, h], qkv[:, 1, h], qkv[:, 2, h])
        heads += 1
        if time.perf_counter() - t0 > budget_s * 0.2:
            break
    t_pre += (time.perf_counter() - t0) * (nh / heads)
    okv = O.KVCache.empty(1, nh, s, dh, bool(kvq), kvq == "h16")
    t0 = time.perf_counter()
    okv.store(0, 0, xs.reshape(1, s, h1), xs.reshape(1, s, h1))
    t_pre += time.perf_counter() - t0
    t_block = sh.l * bls * (t_pre + (n - 1) * t_dec_seq)   # the sequences of a block, one after the other
    return {"value": bls * n / t_block, "unit": "tokens/s", "cores": int(threads), "kind": "oracle",
            "decode_tokens_per_s": 1.0 / (sh.l * t_dec_seq), "measured_s": time.perf_counter() - t_begin,
            "sample": "extrapolated: the numpy oracle (float64, BLAS on %d threads) on ONE layer at the real widths "
                      "(h1=%d, h2=%d, %d heads): decode step of 4 sequences at %d cached rows and prefill of one "
                      "sequence of %d positions, each projection timed on a %d-row slab of its weight matrix, "
                      "attention on the heads that fit the time budget; scaled to full matrices and all heads, "
                      "x%d layers, x%d sequences, %d tokens each" % (threads, h1, h2, nh, rows + 1, s, slab, sh.l,
                                                                    bls, n)}


def run_kv_stress(args, torch, B, synth):
    """64 decode steps of one OPT-175B-shaped layer over a 4-bit cache that already holds 2048 rows of
    N(0,1) keys/values for each of 512 sequences; every step appends one quantized K/V row per
    sequence and attends over all rows so far.  One bench step = those 64 layer steps."""
    shape_name, wq, kvq, ngb, b, ctx, n = WORKLOADS[args.workload]
    sh0 = getattr(synth, shape_name)
    sh = synth.Shape(sh0.h1, sh0.nh, sh0.h2, sh0.vocab, sh0.max_pos, 1, sh0.ln_eps)
    cfg = B.Cfg(sh.h1, sh.nh, sh.h2, sh.vocab, max(sh.max_pos, ctx + n), sh.ln_eps)
    layers, _, _, _, _ = build_model(sh, wq, args.seed, torch, B, embeddings=False)
    w = layers[0]
    kv = B.KVCache(cfg, b, ctx + n, bool(kvq), zero=False, meta_f16=kvq == "h16")
    g = torch.Generator(device="cuda")
    g.manual_seed(args.seed * 1000003 + 77)
    chunk = 256   # rows per fill call: 512 x 256 x 12288 FP16 = 3.2 GB of K and of V at a time
    for r0 in range(0, ctx, chunk):
        r1 = min(ctx, r0 + chunk)
        k = torch.empty((b * (r1 - r0), sh.h1), dtype=torch.float16, device="cuda").normal_(0.0, 1.0, generator=g)
        v = torch.empty((b * (r1 - r0), sh.h1), dtype=torch.float16, device="cuda").normal_(0.0, 1.0, generator=g)
        B.fg_kv_append(cfg, k, v, sh.h1, b, r1 - r0, kv, 0, r0)
        del k, v
    x = torch.empty((b, sh.h1), dtype=torch.float16, device="cuda").normal_(0.0, 1.0, generator=g)
    out = torch.empty_like(x)
    ws = torch.empty(B.lib().fg_layer_workspace_bytes(B.C.byref(cfg.c), B.C.byref(w.c), b), dtype=torch.uint8,
                     device="cuda")
    torch.cuda.synchronize()

    def step():
        for i in range(n):
            B.fg_decode_layer(cfg, w, x, ctx + i, kv, 0, ws=ws, out=out)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    B.fg_profile_begin()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    prof = B.fg_profile_end()
    K = args.steps
    kv_bytes = sum(2.0 * b * sh.h1 * (ctx + i + 1) * bpe(kvq) for i in range(n))
    P = 4 * sh.h1 * sh.h1 + 2 * sh.h1 * sh.h2
    rl = {}
    for name, bound, work in (("attn_decode", "hbm", kv_bytes), ("gemm_large_m", "mfma", 2.0 * b * P * n),
                              ("kv_append", "hbm", n * 2.0 * b * sh.h1 * (2 + bpe(kvq)))):
        if name not in prof:
            continue
        ms = prof[name]["ms"] / K
        peak = HBM_PEAK if bound == "hbm" else MFMA_F16_PEAK
        ach = work / (ms * 1e-3)
        rl[name] = {"bound": bound, "achieved": ach / (1e9 if bound == "hbm" else 1e12),
                    "peak": peak / (1e9 if bound == "hbm" else 1e12), "unit": "GB/s" if bound == "hbm" else "TFLOP/s",
                    "frac": ach / peak, "traffic": None, "ms_per_step": ms,
                    "launches_per_step": prof[name]["launches"] / K,
                    "avg_launch_us": 1e3 * prof[name]["ms"] / prof[name]["launches"]}
    dominant = max(rl, key=lambda k: rl[k]["ms_per_step"])
    line = {
        "metric": "generated tokens/s + % peak HBM BW, 4-bit OPT-175B-shape decode, 1 GPU",
        "value": b * n * K / elapsed, "unit": "tokens/s", "n_gpus": 1, "steps": K, "warmup": args.warmup,
        "ms_per_step": 1e3 * elapsed / K, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16", "data": "synthetic",
        "config": {"workload": args.workload, "shape": {"l": 1, "h1": sh.h1, "nh": sh.nh, "h2": sh.h2},
                   "weights": "q4g64", "kv_cache": "q4g64_h16" if kvq == "h16" else "q4g64", "block": "1x%d" % b, "context": ctx, "decode_steps": n},
        "decode": {"ms_per_layer_step": 1e3 * elapsed / K / n,
                   "hbm_frac_avg": (kv_bytes + n * P * bpe(wq)) / (elapsed / K) / HBM_PEAK},
        "roofline": dict(rl[dominant], kernel=dominant), "roofline_kernels": rl,
        "kernel_ms": {k: v["ms"] / K for k, v in prof.items() if v["launches"]},
    }
    print(json.dumps(line))


def run_diagonal(args, torch, B, synth):
    """The whole queue of ngb x gbs sequences generated in the diagonal order (fg_generate_diagonal):
    one GPU batch admitted per iteration, paged 4-bit caches sized by fg_diagonal_pages_needed."""
    shape_name, wq, kvq, ngb, gbs, s, n = WORKLOADS[args.workload]
    sh = getattr(synth, shape_name)
    if args.layers:
        sh = synth.Shape(sh.h1, sh.nh, sh.h2, sh.vocab, sh.max_pos, args.layers, sh.ln_eps)
    n_seqs = ngb * gbs
    cfg = B.Cfg(sh.h1, sh.nh, sh.h2, sh.vocab, sh.max_pos, sh.ln_eps)
    t_setup = time.time()
    layers, emb, pos, lnf_g, lnf_b = build_model(sh, wq, args.seed, torch, B)
    need = B.fg_diagonal_pages_needed(n_seqs, s, n, gbs)
    pages = [B.KVPages(cfg, need, kvq == "h16", zero=False) for _ in range(sh.l)]
    ws = torch.empty(B.lib().fg_diagonal_workspace_bytes(B.C.byref(cfg.c), B.C.byref(layers[0].c), n_seqs, s, n, gbs),
                     dtype=torch.uint8, device="cuda")
    out_ids = torch.zeros((n_seqs, n), dtype=torch.int32, device="cuda")
    prompt = torch.from_numpy(synth.prompt_ids(n_seqs, s, sh.vocab, args.seed)).cuda()
    torch.cuda.synchronize()
    resident = sum(w.nbytes() for w in layers) + sum(p.nbytes() for p in pages) + emb.numel() * 2 + pos.numel() * 2
    t_setup = time.time() - t_setup

    def step():
        return B.fg_generate_diagonal(cfg, layers, emb, pos, lnf_g, lnf_b, prompt, n, gbs, pages, ws=ws, out_ids=out_ids)

    # the first pass is timed on the host to plan how many passes fit the wall-clock budget
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    if args.warmup == 0:
        B.fg_profile_begin()
    _, st = step()
    torch.cuda.synchronize()
    first_s = time.perf_counter() - t0
    W, K = plan_passes(args.steps, args.warmup, first_s,
                       args.budget_s - (time.perf_counter() - T_PROCESS_START) - 10.0)
    for _ in range(W - 1):
        step()
    torch.cuda.synchronize()
    elapsed = first_s if args.warmup == 0 else 0.0
    if args.warmup != 0:
        B.fg_profile_begin()
    t0 = time.perf_counter()
    for _ in range(K - (1 if args.warmup == 0 else 0)):
        _, st = step()
    torch.cuda.synchronize()
    elapsed += time.perf_counter() - t0
    prof = B.fg_profile_end()
    P = 4 * sh.h1 * sh.h1 + 2 * sh.h1 * sh.h2
    rl = {}
    for name, bound, work in (("gemm_large_m", "mfma", 2.0 * n_seqs * s * P * sh.l),
                              ("gemm_small_m", "mfma", 2.0 * n_seqs * (n - 1) * (sh.l * P + sh.vocab * sh.h1)
                               + 2.0 * n_seqs * sh.vocab * sh.h1),
                              ("attn_decode", "hbm", sum(2.0 * n_seqs * sh.l * sh.h1 * (s + i) * bpe(kvq)
                                                         for i in range(1, n)))):
        if name not in prof:
            continue
        ms = prof[name]["ms"] / K
        peak = HBM_PEAK if bound == "hbm" else MFMA_F16_PEAK
        ach = work / (ms * 1e-3)
        rl[name] = {"bound": bound, "achieved": ach / (1e9 if bound == "hbm" else 1e12),
                    "peak": peak / (1e9 if bound == "hbm" else 1e12), "unit": "GB/s" if bound == "hbm" else "TFLOP/s",
                    "frac": ach / peak, "traffic": None, "ms_per_step": ms,
                    "launches_per_step": prof[name]["launches"] / K,
                    "avg_launch_us": 1e3 * prof[name]["ms"] / prof[name]["launches"]}
    dominant = max(rl, key=lambda k: rl[k]["ms_per_step"])
    block_pages = n_seqs * -(-(s + n) // B.PAGE_ROWS)
    line = {
        "metric": "generated tokens/s + % peak HBM BW, 4-bit OPT-175B-shape decode, 1 GPU",
        "value": n_seqs * n * K / elapsed, "unit": "tokens/s", "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": 1e3 * elapsed / K, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16", "data": "synthetic",
        "config": {"workload": args.workload + ("" if not args.layers else "_%dlayers" % args.layers),
                   "shape": {"l": sh.l, "h1": sh.h1, "nh": sh.nh, "h2": sh.h2, "vocab": sh.vocab},
                   "weights": "q4g64_h16" if wq == "h16" else "q4g64",
                   "kv_cache": "paged " + ("q4g64_h16" if kvq == "h16" else "q4g64"), "schedule": "diagonal",
                   "sequences": n_seqs, "admitted_per_iteration": gbs, "iterations": ngb + n - 1,
                   "prompt_len": s, "gen_len": n, "resident_gb": resident / 1e9, "setup_s": t_setup,
                   "peak_pages_per_layer": st["peak_pages"], "block_schedule_pages_per_layer": block_pages},
        "roofline": dict(rl[dominant], kernel=dominant), "roofline_kernels": rl,
        "kernel_ms": {k: v["ms"] / K for k, v in prof.items() if v["launches"]},
    }
    print(json.dumps(line))


def roofline_table(prof, alg, passes, small_flops, small_bytes):
    """Per kernel class: algorithmic work / summed event time.  alg: {class: (bound, work per pass)}."""
    rl = {}
    for name, (bound, work) in alg.items():
        if name not in prof:
            continue
        ms = prof[name]["ms"] / passes
        launches = prof[name]["launches"]
        if name == "gemm_small_m" and "gemm_small_m_finish" in prof:
            ms += prof["gemm_small_m_finish"]["ms"] / passes      # the reduction pass belongs to the projection
        peak = HBM_PEAK if bound == "hbm" else MFMA_F16_PEAK
        ach = work / (ms * 1e-3)
        rl[name] = {"bound": bound, "achieved": ach / 1e9 if bound == "hbm" else ach / 1e12,
                    "peak": peak / 1e9 if bound == "hbm" else peak / 1e12,
                    "unit": "GB/s" if bound == "hbm" else "TFLOP/s", "frac": ach / peak, "traffic": None,
                    "ms_per_step": ms, "launches_per_step": launches / passes,
                    "avg_launch_us": 1e3 * ms * passes / launches}
    if "gemm_small_m" in rl:
        # The decode projections stream every weight once (HBM bound) and do 2*bls flops per weight
        # (MFMA bound): the roofline is whichever takes longer at this block size; both fractions are kept.
        r = rl["gemm_small_m"]
        ms = r["ms_per_step"]
        r["includes"] = "gemm_small_m_finish (reduction pass of the split contraction)"
        r["hbm_frac"] = small_bytes / (ms * 1e-3) / HBM_PEAK
        r["mfma_frac"] = small_flops / (ms * 1e-3) / MFMA_F16_PEAK
        if small_flops / MFMA_F16_PEAK > small_bytes / HBM_PEAK:
            r.update(bound="mfma", achieved=small_flops / (ms * 1e-3) / 1e12, peak=MFMA_F16_PEAK / 1e12,
                     unit="TFLOP/s", frac=r["mfma_frac"])
    return rl


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5, help="timed passes, at most (see --budget-s)")
    ap.add_argument("--warmup", type=int, default=1, help="warm-up passes, at most")
    ap.add_argument("--budget-s", type=float, default=400.0,
                    help="wall-clock budget of the whole run in seconds, counted from process start")
    ap.add_argument("--workload", default="opt175b_q4", choices=sorted(WORKLOADS))
    ap.add_argument("--layers", type=int, default=0, help="override the layer count (debugging only; marks the line)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-kernel-table", action="store_true", help="skip the extra pass with events on every launch")
    ap.add_argument("--seed", type=int, default=0)
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no sharding or collectives); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2303_06865_amd import binding as B
    from paper_2303_06865_amd import synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    B.lib()   # fails loudly if the HIP library is not built
    torch.cuda.set_device(0)

    if args.workload.startswith("kv_stress"):
        return run_kv_stress(args, torch, B, synth)
    if args.workload.endswith("_diagonal"):
        return run_diagonal(args, torch, B, synth)
    shape_name, wq, kvq, ngb, gbs, s, n = WORKLOADS[args.workload]
    sh = getattr(synth, shape_name)
    if args.layers:
        sh = synth.Shape(sh.h1, sh.nh, sh.h2, sh.vocab, sh.max_pos, args.layers, sh.ln_eps)
    bls = ngb * gbs
    cfg = B.Cfg(sh.h1, sh.nh, sh.h2, sh.vocab, sh.max_pos, sh.ln_eps)

    t_setup = time.time()
    layers, emb, pos, lnf_g, lnf_b = build_model(sh, wq, args.seed, torch, B)
    cap = s + n
    kv = [B.KVCache(cfg, bls, cap, bool(kvq), zero=False, meta_f16=kvq == "h16") for _ in range(sh.l)]
    ws = torch.empty(B.fg_workspace_bytes(cfg, layers[0], gbs, ngb, s), dtype=torch.uint8, device="cuda")
    out_ids = torch.zeros((bls, n), dtype=torch.int32, device="cuda")
    prompt = torch.from_numpy(synth.prompt_ids(bls, s, sh.vocab, args.seed)).cuda()
    torch.cuda.synchronize()
    resident = sum(w.nbytes() for w in layers) + sum(k.nbytes() for k in kv) + emb.numel() * 2 + pos.numel() * 2
    t_setup = time.time() - t_setup
    print("bench.py: %s resident after %.1f s of set-up" % (args.workload, t_setup), file=sys.stderr, flush=True)

    def one_pass():
        """One step of the benchmark: fg_generate over the block; returns (stats, wall seconds)."""
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        st = B.fg_generate(cfg, layers, emb, pos, lnf_g, lnf_b, prompt, n, ngb, gbs, kv, ws=ws, out_ids=out_ids,
                           want_stats=True)[1]
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        # progress on stderr (stdout carries the one JSON line): a pass of the headline workload takes
        # about 25 s, and a harness that watches for output must not take the run for hung
        print("bench.py: pass done in %.2f s (%.0f s since start)" % (dt, time.perf_counter() - T_PROCESS_START),
              file=sys.stderr, flush=True)
        return st, dt

    # ---- first pass (warm-up if one was asked for), then plan what still fits the budget
    timed_cheap = list(CHEAP_TO_TIME)
    stats, walls = [], []
    if args.warmup == 0:
        B.fg_profile_begin(timed_cheap)
    st, first_s = one_pass()
    if args.warmup == 0:
        stats.append(st)
        walls.append(first_s)
    reserve = (0.0 if args.no_kernel_table else 1.25 * first_s) + (0.0 if args.no_cpu_baseline else 35.0) + 5.0
    avail = args.budget_s - (time.perf_counter() - T_PROCESS_START) - reserve
    W, K = plan_passes(args.steps, args.warmup, first_s, avail)
    for _ in range(W - 1):
        one_pass()
    # ---- timed region: K passes, events only on the few long prefill launches
    if args.warmup != 0:
        B.fg_profile_begin(timed_cheap)
    while len(stats) < K:
        st, w = one_pass()
        stats.append(st)
        walls.append(w)
    prof_timed = B.fg_profile_end()
    elapsed = sum(walls)

    tokens = bls * n * K
    value = tokens / elapsed
    prefill_s = sum(st["prefill_s"] for st in stats) / K
    decode_s = sum(st["decode_s"] for st in stats) / K
    step_s = [sum(st["decode_step_s"][i] for st in stats) / K for i in range(n - 1)]

    # ---- one extra pass with events on every launch: the per-kernel-class table (not part of `value`)
    prof_all, evented = None, None
    if not args.no_kernel_table:
        B.fg_profile_begin()
        st, w = one_pass()
        prof_all = B.fg_profile_end()
        evented = {"wall_s": w, "prefill_s": st["prefill_s"], "decode_s": st["decode_s"]}

    # ---- algorithmic bytes / flops of each kernel class per generate (Section 4.3 terms, re-priced)
    P = 4 * sh.h1 * sh.h1 + 2 * sh.h1 * sh.h2
    w_bytes = sh.l * P * bpe(wq)
    head_bytes = sh.vocab * sh.h1 * 2.0
    kv_bytes = [2.0 * bls * sh.l * sh.h1 * (s + i) * bpe(kvq) for i in range(1, n)]
    small_bytes = (n - 1) * (w_bytes + head_bytes) + head_bytes
    alg = {
        "gemm_large_m": ("mfma", 2.0 * bls * s * P * sh.l),
        "attn_prefill": ("mfma", 4.0 * bls * s * s * sh.h1 * sh.l / 2.0),
        "attn_decode": ("hbm", float(sum(kv_bytes))),
        "gemm_small_m": ("hbm", small_bytes),
        "kv_append": ("hbm", (2.0 * bls * s * sh.h1 * (2.0 + bpe(kvq)) + (n - 1) * 2.0 * bls * sh.h1 * (2 + bpe(kvq))) * sh.l),
    }
    small_flops = 2.0 * bls * ((n - 1) * (sh.l * P + sh.vocab * sh.h1) + sh.vocab * sh.h1)
    rl_timed = roofline_table(prof_timed, alg, K, small_flops, small_bytes)
    rl_all = roofline_table(prof_all, alg, 1, small_flops, small_bytes) if prof_all else {}
    for k, v in rl_timed.items():
        v["measured_in"] = "the %d timed passes" % K
    for k, v in rl_all.items():
        v["measured_in"] = "one extra pass with events on every launch"
    table = dict(rl_all)
    table.update(rl_timed)     # where both exist, the figure taken over the timed region wins
    dominant = max(table, key=lambda k: table[k]["ms_per_step"]) if table else None
    # HBM traffic per launch comes from rocprofv3 counter runs (it cannot be measured from inside this
    # process); the summaries under profiles/ and the file that collects their figures say when and how
    traffic_file = os.path.join(ROOT, "profiles", "traffic.json")
    if os.path.exists(traffic_file):
        try:
            tr = json.load(open(traffic_file))
            for k, v in tr.get(args.workload, {}).items():
                if k in table:
                    table[k]["traffic"] = v
                    table[k]["traffic_source"] = tr.get("_source", "profiles/traffic.json (rocprofv3 --pmc runs)")
        except Exception:
            pass

    decode = {}
    if n > 1:
        pick = sorted(set([0, (n - 1) // 2, n - 2]))
        decode = {
            "tokens_per_s": bls * (n - 1) / decode_s,
            "ms_per_token_step": 1e3 * decode_s / (n - 1),
            "hbm_frac_avg": (w_bytes + sum(kv_bytes) / (n - 1)) / (decode_s / (n - 1)) / HBM_PEAK,
            "hbm_frac_at_step": {str(i + 1): (w_bytes + kv_bytes[i]) / step_s[i] / HBM_PEAK for i in pick},
            "bytes_per_step_avg": w_bytes + sum(kv_bytes) / (n - 1),
            "note": "timed passes: no per-launch events on the decode kernels",
        }

    line = {
        "metric": "generated tokens/s + % peak HBM BW, 4-bit OPT-175B-shape decode, 1 GPU",
        "value": value, "unit": "tokens/s", "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": 1e3 * elapsed / K, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16", "data": "synthetic",
        "config": {"workload": args.workload + ("" if not args.layers else "_%dlayers" % args.layers),
                   "shape": {"l": sh.l, "h1": sh.h1, "nh": sh.nh, "h2": sh.h2, "vocab": sh.vocab},
                   "weights": "q4g64_h16" if wq == "h16" else ("q4g64" if wq else "f16"), "kv_cache": "q4g64_h16" if kvq == "h16" else ("q4g64" if kvq else "f16"),
                   "block": "%dx%d" % (ngb, gbs), "prompt_len": s, "gen_len": n,
                   "resident_gb": resident / 1e9, "setup_s": t_setup,
                   "requested": {"steps": args.steps, "warmup": args.warmup, "budget_s": args.budget_s},
                   "first_pass_s": first_s},
        "prefill_s": prefill_s, "decode_s": decode_s, "decode": decode,
        "roofline": (dict(table[dominant], kernel=dominant) if dominant else None),
        "roofline_kernels": table,
        "kernel_ms": {k: v["ms"] for k, v in (prof_all or prof_timed).items() if v["launches"]},
        "evented_pass": evented,
        "paper_context": "FlexGen reports 1.12 token/s for OPT-175B (4-bit) on one 16 GB T4 with CPU offloading",
    }
    if not args.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(sh, wq, kvq, s, n, bls)
    line["wall_s"] = time.perf_counter() - T_PROCESS_START
    print(json.dumps(line))


if __name__ == "__main__":
    main()
