"""Single-kernel timing harness: runs ONE kernel class at one shape through the C ABI and prints one
JSON line with its average launch duration (from the library's own HIP-event profile) and the
algorithmic bytes / flops per launch.  It exists so that `rocprofv3 --kernel-trace --stats` and
`rocprofv3 --pmc ...` can be pointed at a single kernel at the shape the benchmark runs it at:

  python3 kernel_bench.py linear --m 144 --n 36864 --k 12288 --wdtype q4t
  python3 kernel_bench.py attn_decode --batch 144 --nh 96 --rows 528
  python3 kernel_bench.py attn_decode_topk --batch 144 --nh 96 --rows 528 --topk 53
  python3 kernel_bench.py attn_decode_paged --batch 144 --nh 96 --rows 528
  python3 kernel_bench.py attn_prefill --batch 8 --nh 96 --seq 512
  python3 kernel_bench.py copy --mib 1024      # calibration for HBM counters

Inputs are seeded synthetic tensors generated on the device (weights ~ N(0, 0.02), activations
~ N(0, 1), cache codes uniform), i.e. the value distributions of the benchmark's model builder.
"""
import argparse
import json
import os
import sys

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import torch

from paper_2303_06865_amd import binding as B


def _time_classes(fn, iters, warm):
    for _ in range(warm):
        fn()
    torch.cuda.synchronize()
    B.fg_profile_begin()
    for _ in range(iters):
        fn()
    prof = B.fg_profile_end()
    return {k: {"ms": v["ms"] / iters, "launches": v["launches"] / iters} for k, v in prof.items() if v["launches"]}


def _torch_time(fn, iters, warm):
    for _ in range(warm):
        fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(iters):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / iters


def main(argv=None):
    ap = argparse.ArgumentParser()
    ap.add_argument("op", choices=["linear", "attn_decode", "attn_decode_topk", "attn_decode_paged", "attn_prefill",
                                   "copy"])
    ap.add_argument("--m", type=int, default=144)
    ap.add_argument("--n", type=int, default=36864)
    ap.add_argument("--k", type=int, default=12288)
    ap.add_argument("--wdtype", choices=["f16", "q4", "q4t", "q4th"], default="q4t",
                    help="weight storage: FP16, 4-bit canonical, 4-bit tiled, 4-bit tiled with FP16 pairs")
    ap.add_argument("--batch", type=int, default=144)
    ap.add_argument("--nh", type=int, default=96)
    ap.add_argument("--dh", type=int, default=128)
    ap.add_argument("--rows", type=int, default=528, help="cached positions read by decode attention")
    ap.add_argument("--cap", type=int, default=0, help="attn_decode*: cache capacity in positions (default rows + 64)")
    ap.add_argument("--seq", type=int, default=512)
    ap.add_argument("--topk", type=int, default=0, help="attn_decode_topk: rows kept (default: ceil(rows / 10))")
    ap.add_argument("--kv", choices=["q4", "q4h", "f16"], default="q4", help="cache storage: 4-bit, 4-bit with FP16 pairs, FP16")
    ap.add_argument("--mib", type=int, default=1024, help="copy: MiB read (and as many written)")
    ap.add_argument("--iters", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    a = ap.parse_args(argv)

    torch.manual_seed(0)
    dev = "cuda"
    out = {"op": a.op}
    if a.op == "linear":
        w = torch.randn(a.n, a.k, device=dev, dtype=torch.float16) * 0.02
        mat = B.Mat.from_f16(w, a.wdtype != "f16", tiled=a.wdtype in ("q4t", "q4th"), meta_f16=a.wdtype == "q4th")
        del w
        x = torch.randn(a.m, a.k, device=dev, dtype=torch.float16)
        out.update(m=a.m, n=a.n, k=a.k, wdtype=a.wdtype,
                   bytes=int(a.n * a.k * {"f16": 2, "q4th": 0.5625}.get(a.wdtype, 0.625)), flops=2 * a.m * a.n * a.k)
        out["classes"] = _time_classes(lambda: B.fg_linear(mat, None, x), a.iters, a.warmup)
    elif a.op in ("attn_decode", "attn_decode_topk"):
        h1 = a.nh * a.dh
        cfg = B.Cfg(h1, a.nh, 4 * h1, 50272, 4096)
        q4 = a.kv != "f16"
        kvb = {"q4": 0.625, "q4h": 0.5625, "f16": 2.0}[a.kv]
        kv = B.KVCache(cfg, a.batch, a.cap or a.rows + 64, q4, zero=False, meta_f16=a.kv == "q4h")
        if q4:
            kv.k_codes.random_(0, 256)
            kv.v_codes.random_(0, 256)
            kv.k_meta.copy_(torch.randn(kv.k_meta.shape, device=dev).abs_().mul_(0.3))
            kv.v_meta.copy_(torch.randn(kv.v_meta.shape, device=dev).abs_().mul_(0.3))
        else:
            kv.k_codes.normal_()
            kv.v_codes.normal_()
        qkv = torch.randn(a.batch, 3 * h1, device=dev, dtype=torch.float16)
        if a.op == "attn_decode_topk":
            topk = a.topk or -(-a.rows // 10)
            # K stream in full, topk rows of V
            out.update(batch=a.batch, nh=a.nh, dh=a.dh, rows=a.rows, topk=topk, kv=a.kv,
                       bytes=int(a.batch * a.nh * (a.rows + topk) * a.dh * kvb),
                       flops=2 * a.batch * a.nh * (a.rows + topk) * a.dh)
            out["classes"] = _time_classes(
                lambda: B.fg_decode_attention_topk(cfg, qkv, 3 * h1, a.batch, a.rows, topk, kv, 0), a.iters, a.warmup)
        else:
            out.update(batch=a.batch, nh=a.nh, dh=a.dh, rows=a.rows, kv=a.kv,
                       bytes=int(2 * a.batch * a.nh * a.rows * a.dh * kvb),
                       flops=4 * a.batch * a.nh * a.rows * a.dh)
            out["classes"] = _time_classes(lambda: B.fg_decode_attention(cfg, qkv, 3 * h1, a.batch, a.rows, kv, 0),
                                           a.iters, a.warmup)
    elif a.op == "attn_decode_paged":
        # every sequence `rows` long, its pages scattered over the pool by a random permutation
        h1 = a.nh * a.dh
        cfg = B.Cfg(h1, a.nh, 4 * h1, 50272, 4096)
        h16 = a.kv == "q4h"
        assert a.kv != "f16", "pages hold 4-bit rows only"
        kvb = 0.5625 if h16 else 0.625
        per_seq = -(-a.rows // B.PAGE_ROWS)
        n_pages = a.batch * per_seq
        pages = B.KVPages(cfg, n_pages, h16, zero=False)
        pages.k_codes.random_(0, 256)
        pages.v_codes.random_(0, 256)
        pages.k_meta.copy_(torch.randn(pages.k_meta.shape, device=dev).abs_().mul_(0.3))
        pages.v_meta.copy_(torch.randn(pages.v_meta.shape, device=dev).abs_().mul_(0.3))
        table = torch.randperm(n_pages, device=dev).to(torch.int32).reshape(a.batch, per_seq).contiguous()
        seqs = B.Ragged(table, None, torch.full((a.batch,), a.rows, dtype=torch.int32, device=dev))
        qkv = torch.randn(a.batch, 3 * h1, device=dev, dtype=torch.float16)
        out.update(batch=a.batch, nh=a.nh, dh=a.dh, rows=a.rows, kv=a.kv,
                   bytes=int(2 * a.batch * a.nh * a.rows * a.dh * kvb), flops=4 * a.batch * a.nh * a.rows * a.dh)
        out["classes"] = _time_classes(lambda: B.fg_decode_attention_paged(cfg, qkv, 3 * h1, a.batch, pages, seqs, 0),
                                       a.iters, a.warmup)
    elif a.op == "attn_prefill":
        h1 = a.nh * a.dh
        cfg = B.Cfg(h1, a.nh, 4 * h1, 50272, 4096)
        qkv = torch.randn(a.batch * a.seq, 3 * h1, device=dev, dtype=torch.float16)
        out.update(batch=a.batch, nh=a.nh, dh=a.dh, seq=a.seq, bytes=int(4 * a.batch * a.seq * h1 * 2),
                   flops=4 * a.batch * a.nh * a.seq * a.seq * a.dh // 2)
        out["classes"] = _time_classes(lambda: B.fg_prefill_attention(cfg, qkv, a.batch, a.seq), a.iters, a.warmup)
    else:
        n = a.mib << 20
        # a streaming elementwise kernel (a same-dtype tensor copy may be served by a DMA engine and
        # would then not show up in per-kernel counters): reads n bytes, writes n bytes
        src = torch.randn(n // 4, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        ms = _torch_time(lambda: torch.add(src, 1.0, out=dst), a.iters, a.warmup)
        out.update(bytes_read=n, bytes_written=n, ms=ms, tbps=2 * n / ms / 1e9)
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
