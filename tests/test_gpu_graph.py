"""The decode layer under HIP graph capture.

The library allocates nothing, clears nothing with memset nodes and synchronises nothing, so a caller
can record a decode step into a graph and replay it (Algorithm 1's inner loop is launch-bound for small
models).  The test records `fg_decode_layer` of a small 4-bit model into a graph and replays it several
times, with eager work and synchronisations of the program between the replays, and checks every replay
bit for bit against the eager call on the same inputs: the same kernels on the same data in the same
order must give the same bits, and the cache row the step appends must be the eager one.
"""
import numpy as np
import pytest
import torch

from paper_2303_06865_amd import binding as B
from paper_2303_06865_amd import synth

from util import cfg_pair, dev, host

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("quant_w,tiled,quant_kv,b", [(True, True, True, 4), (True, True, True, 80), (False, False, False, 16)])
def test_decode_layer_replayed_from_a_graph_equals_eager(quant_w, tiled, quant_kv, b):
    sh = synth.Shape(h1=768, nh=12, h2=3072, vocab=2048, max_pos=64)
    _, cfg = cfg_pair(sh)
    t = synth.layer_tensors(sh, 11, 0, std=0.02, biases=True, random_ln=True)
    w = B.LayerWeights.from_numpy(t, quant_w, tiled=tiled)
    s = 9
    x0 = synth.activations_f16((b, s, sh.h1), 0.05, 3)

    def fresh_cache():
        kv = B.KVCache(cfg, b, s + 4, quant_kv)
        B.fg_prefill_layer(cfg, w, dev(x0), kv)
        return kv

    n_ws = B.lib().fg_layer_workspace_bytes(B.C.byref(cfg.c), B.C.byref(w.c), b)
    inputs = [synth.activations_f16((b, sh.h1), 0.05, 100 + i) for i in range(4)]

    # eager results, each from a cache in the state the graph's cache will be in (prompt rows only)
    eager = []
    for xi in inputs:
        kv_e = fresh_cache()
        out = B.fg_decode_layer(cfg, w, dev(xi), s, kv_e)
        torch.cuda.synchronize()
        eager.append((host(out).view(np.uint16).copy(), host(kv_e.k_codes).copy(), host(kv_e.v_codes).copy()))

    kv = fresh_cache()
    x_static = dev(inputs[0]).clone()
    out_static = torch.empty_like(x_static)
    ws = torch.empty(max(n_ws, 16), dtype=torch.uint8, device="cuda")
    # warm-up outside the capture: first launches set kernel attributes, which is not stream work
    B.fg_decode_layer(cfg, w, x_static, s, kv, ws=ws, out=out_static)
    torch.cuda.synchronize()

    g = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(g, stream=side):
            B.fg_decode_layer(cfg, w, x_static, s, kv, ws=ws, out=out_static)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()

    for rep, xi in enumerate(inputs):
        x_static.copy_(dev(xi))
        # eager work of the program and a synchronisation between the replays
        junk = torch.randn(1 << 16, device="cuda").sum().item()
        assert np.isfinite(junk)
        g.replay()
        torch.cuda.synchronize()
        want_out, want_k, want_v = eager[rep]
        assert np.array_equal(host(out_static).view(np.uint16), want_out), "replay %d: output differs from the eager call" % rep
        assert np.array_equal(host(kv.k_codes), want_k) and np.array_equal(host(kv.v_codes), want_v), "replay %d: cache" % rep


def _table(lens, n_pages, stride, seed):
    """Pages handed to sequences in a shuffled order: ceil(len / 64) each, -1 in the unused slots."""
    perm = np.random.default_rng(seed).permutation(n_pages)
    table = np.full((len(lens), stride), -1, np.int32)
    nxt = 0
    for q, ln in enumerate(lens):
        for slot in range(-(-ln // 64)):
            table[q, slot] = perm[nxt]
            nxt += 1
    assert nxt <= n_pages
    return table


@pytest.mark.parametrize("meta_f16", [False, True])
def test_one_paged_graph_serves_every_token_step(meta_f16):
    """The paged step reads each row's position from device memory, so one recorded graph serves a whole
    generation loop: between replays the program adds one to the positions on the device and writes the
    next input.  Six ragged steps (rows cross a page boundary at different steps) from one graph against
    six eager calls on a second pool: outputs and all four page arrays equal bit for bit at every step."""
    sh = synth.Shape(h1=768, nh=12, h2=3072, vocab=2048, max_pos=256)
    _, cfg = cfg_pair(sh)
    t = synth.layer_tensors(sh, 5, 0, std=0.02, biases=True, random_ln=True)
    w = B.LayerWeights.from_numpy(t, True, tiled=True)
    steps = 6
    lens = [61, 3, 64, 125, 17]                          # prompt rows per sequence
    n_seqs, s_max = len(lens), max(lens)
    table = dev(_table([ln + steps for ln in lens], 12, 3, seed=4))
    order = dev(np.array([2, 0, 4, 1, 3], np.int32))     # the step's rows name the sequences in this order
    pos0 = dev(np.array([lens[q] for q in [2, 0, 4, 1, 3]], np.int32))

    def filled_pool():
        pages = B.KVPages(cfg, 12, meta_f16)
        for q, ln in enumerate(lens):                    # one prefill per length: prompts are not padded
            xq = synth.activations_f16((1, ln, sh.h1), 0.05, 40 + q)
            B.fg_prefill_layer_paged(cfg, w, dev(xq), pages, B.Ragged(table, dev(np.array([q], np.int32)), None))
        return pages

    inputs = [synth.activations_f16((n_seqs, sh.h1), 0.05, 200 + i) for i in range(steps)]
    n_ws = B.lib().fg_layer_workspace_bytes(B.C.byref(cfg.c), B.C.byref(w.c), n_seqs)
    ws = torch.empty(max(n_ws, 16), dtype=torch.uint8, device="cuda")

    def pool_bits(p):
        bits = np.uint16 if meta_f16 else np.uint32
        return (host(p.k_codes).copy(), host(p.v_codes).copy(), host(p.k_meta).view(bits).copy(), host(p.v_meta).view(bits).copy())

    eager_pages = filled_pool()
    eager = []
    for i, xi in enumerate(inputs):
        out = B.fg_decode_layer_paged(cfg, w, dev(xi), eager_pages, B.Ragged(table, order, pos0 + i), ws=ws)
        torch.cuda.synchronize()
        eager.append((host(out).view(np.uint16).copy(), pool_bits(eager_pages)))

    pages = filled_pool()
    pos = pos0.clone()
    seqs = B.Ragged(table, order, pos)
    x_static = dev(inputs[0]).clone()
    out_static = torch.empty_like(x_static)
    torch.cuda.synchronize()

    g = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(g, stream=side):
            B.fg_decode_layer_paged(cfg, w, x_static, pages, seqs, ws=ws, out=out_static)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()

    for i, xi in enumerate(inputs):
        x_static.copy_(dev(xi))
        junk = torch.randn(1 << 16, device="cuda").sum().item()
        assert np.isfinite(junk)
        g.replay()
        torch.cuda.synchronize()
        want_out, want_pool = eager[i]
        assert np.array_equal(host(out_static).view(np.uint16), want_out), "step %d: output differs from the eager call" % i
        for name, a, e in zip(("k codes", "v codes", "k meta", "v meta"), pool_bits(pages), want_pool):
            assert np.array_equal(a, e), "step %d: %s differ from the eager pool" % (i, name)
        pos.add_(1)                                      # in place: the graph holds this buffer's address
