"""Pins for the oracle's model-level pieces: the paper's printed memory figures,
cost-model terms, schedule invariants of the block schedule (Algorithm 1) and
the greedy rule."""
import os

import numpy as np
import pytest

from oracle import fg_oracle as O
from paper_2303_06865_amd import synth

GOLD = os.path.join(os.path.dirname(__file__), "golden", "paper_memory_analysis.txt")


def _gold():
    out = {}
    for line in open(GOLD):
        if line.startswith("#") or not line.strip():
            continue
        k, v = line.split()[:2]
        out[k] = float(v)
    return out


def test_memory_analysis_matches_paper_figures():
    """Section 3: OPT-175B FP16 weights '325 GB'; KV cache at b=512, s=512, n=32
    '1.2 TB', '3.8x' the weights.  The printed units are binary multiples."""
    g = _gold()
    w = O.weight_bytes_fp16(96, 12288, 49152)
    kv = O.kv_bytes_fp16_peak(512, 96, 12288, 512, 32)
    assert w == 96 * (8 * 12288 ** 2 + 4 * 12288 * 49152) == 347_892_350_976
    assert abs(w / 2 ** 30 - g["weights_fp16_175b"]) <= 1.0
    assert abs(kv / 2 ** 40 - g["kv_fp16_b512_s512_n32"]) <= 0.05
    assert abs(kv / w - g["kv_over_weights"]) <= 0.05


def test_decode_step_bytes_175b_q4():
    """Config of the headline metric: 96 layers, 144 sequences, 4-bit weights and
    cache.  Weight term = FP16 bytes * 0.625/2; KV term averaged over the 31
    decode steps (rows attended 513..543) = cost-model average s + n/2."""
    w_q4 = O.weight_bytes_fp16(96, 12288, 49152) * 0.625 / 2
    assert abs(w_q4 - 108.7e9) < 0.1e9
    steps = [O.decode_step_bytes(96, 12288, 49152, 144, 512 + i, True, True) for i in range(1, 32)]
    avg = sum(steps) / len(steps)
    assert abs(avg - 220.8e9) < 0.5e9
    kv_avg_formula = 4 * 144 * (512 + 32 / 2) * 12288 * 96 * 0.625 / 2   # Section 4.3: 4 bls (s+n/2) h1 per layer
    assert abs((avg - w_q4) - kv_avg_formula) / kv_avg_formula < 1e-9


def test_flop_terms():
    assert O.decode_linear_flops(1, 12288, 49152, 144) == 144 * (8 * 12288 ** 2 + 4 * 12288 * 49152)
    assert O.prefill_flops(1, 8, 16, 2, 4) == 2 * (8 * 4 * 64 + 4 * 4 * 8 * 16) + 4 * 2 * 16 * 8


def test_greedy_lowest_index_on_ties():
    lg = np.array([[0.0, 3.0, 3.0, 1.0], [5.0, 5.0, 5.0, 5.0], [-1.0, -2.0, -0.5, -0.5]], np.float32)
    assert list(O.greedy(lg)) == [1, 0, 2]


def test_embed_adds_position_rows():
    e = np.arange(12, dtype=np.float16).reshape(4, 3)
    p = (np.arange(6, dtype=np.float16).reshape(2, 3)) * np.float16(0.5)
    x = O.embed(np.array([[3, 0]]), np.array([[0, 1]]), e, p)
    assert np.array_equal(x[0, 0], e[3] + p[0]) and np.array_equal(x[0, 1], e[0] + p[1])


def _tiny_model(l=2, quant=True, seed=0):
    sh = synth.Shape(h1=128, nh=2, h2=256, vocab=211, max_pos=32, l=l)
    cfg = O.ModelCfg(sh.h1, sh.nh, sh.h2, sh.vocab, sh.max_pos)
    layers = []
    for j in range(l):
        t = synth.layer_tensors(sh, seed, j, std=0.08, biases=True, random_ln=True)
        layers.append(O.LayerWeights(
            wqkv=O.Mat.from_f16(t["wqkv"], quant), wo=O.Mat.from_f16(t["wo"], quant),
            w1=O.Mat.from_f16(t["w1"], quant), w2=O.Mat.from_f16(t["w2"], quant),
            ln1_g=t["ln1_g"], ln1_b=t["ln1_b"], ln2_g=t["ln2_g"], ln2_b=t["ln2_b"],
            bqkv=t["bqkv"], bo=t["bo"], b1=t["b1"], b2=t["b2"]))
    m = synth.model_tensors(sh, seed, std=0.08)
    return sh, cfg, layers, m


@pytest.mark.parametrize("quant", [False, True])
def test_block_factorisation_does_not_change_tokens(quant):
    """Sequences of a block are independent, so ids depend neither on how the
    block is cut into GPU batches nor on the neighbours in the batch."""
    sh, cfg, layers, m = _tiny_model(quant=quant)
    prompt = synth.prompt_ids(4, 5, sh.vocab, 1)
    a = O.generate(cfg, layers, m["embed"], m["pos"], m["lnf_g"], m["lnf_b"], prompt, 4, 1, 4, quant)
    b = O.generate(cfg, layers, m["embed"], m["pos"], m["lnf_g"], m["lnf_b"], prompt, 4, 4, 1, quant)
    c = O.generate(cfg, layers, m["embed"], m["pos"], m["lnf_g"], m["lnf_b"], prompt, 4, 2, 2, quant)
    assert a.shape == (4, 4) and a.dtype == np.int32
    assert np.array_equal(a, b) and np.array_equal(a, c)
    solo = O.generate(cfg, layers, m["embed"], m["pos"], m["lnf_g"], m["lnf_b"], prompt[2:3], 4, 1, 1, quant)
    assert np.array_equal(solo[0], a[2])


def test_generate_prefix_property_and_first_token():
    """Generating n tokens then is a prefix of generating n+2; token 1 is the
    argmax of the prefill's last-position logits."""
    sh, cfg, layers, m = _tiny_model(quant=True)
    prompt = synth.prompt_ids(2, 6, sh.vocab, 2)
    a = O.generate(cfg, layers, m["embed"], m["pos"], m["lnf_g"], m["lnf_b"], prompt, 3, 1, 2, True)
    b, logits, caches = O.generate(cfg, layers, m["embed"], m["pos"], m["lnf_g"], m["lnf_b"], prompt, 5, 1, 2, True,
                                   return_trace=True)
    assert np.array_equal(a, b[:, :3])
    # first token by hand: prefill both layers, final LN, tied head
    x = O.embed(prompt, np.broadcast_to(np.arange(6), (2, 6)), m["embed"], m["pos"])
    for j in range(2):
        x = O.prefill_layer(cfg, layers[j], x, O.KVCache.empty(2, sh.nh, 11, sh.dh, True))
    lg = O.lm_head_logits(cfg, x[:, -1], m["lnf_g"], m["lnf_b"], m["embed"])
    assert np.array_equal(lg, logits[0]) and np.array_equal(O.greedy(lg), b[:, 0])
    # the cache holds s + n - 1 rows: the last generated token is never fed back
    assert np.any(caches[0].k_codes[:, :, 6 + 5 - 2] != 0) and np.all(caches[0].k_codes[:, :, 6 + 5 - 1] == 0)


def test_decode_step_uses_absolute_position():
    """Feeding token id at decode step i uses position row s+i-1: changing a
    later position row must not change earlier tokens."""
    sh, cfg, layers, m = _tiny_model(quant=False)
    prompt = synth.prompt_ids(1, 4, sh.vocab, 3)
    a = O.generate(cfg, layers, m["embed"], m["pos"], m["lnf_g"], m["lnf_b"], prompt, 4, 1, 1, False)
    pos2 = m["pos"].copy()
    pos2[5] += np.float16(1.0)       # position of the token fed at step i=2 (0-based) is s+i-1 = 5
    b = O.generate(cfg, layers, m["embed"], pos2, m["lnf_g"], m["lnf_b"], prompt, 4, 1, 1, False)
    assert np.array_equal(a[:, :2], b[:, :2])
    pos3 = m["pos"].copy()
    pos3[7:] += np.float16(1.0)      # rows >= s+n-1 are never read
    c = O.generate(cfg, layers, m["embed"], pos3, m["lnf_g"], m["lnf_b"], prompt, 4, 1, 1, False)
    assert np.array_equal(a, c)


# ---------------------------------------------------------------- LM head (final LN + tied head)
def test_lm_head_logits_against_torch_float64():
    """Independent formulation with library routines: torch.nn.functional.layer_norm in float64,
    FP16 storage of the normalised row, then a float64 matmul against the SAME matrix that embeds the
    tokens (tied head).  A missing final LayerNorm, a swapped gamma/beta, a transposed head or a head
    that is not the embedding fails here."""
    import torch
    rng = np.random.default_rng(11)
    cfg = O.ModelCfg(h1=64, nh=1, h2=128, vocab=37, max_pos=8)
    x = (rng.standard_normal((5, 64)) * 3.0 + 0.7).astype(np.float16)       # non-zero mean: LN must centre it
    g = (1.0 + 0.3 * rng.standard_normal(64)).astype(np.float16)
    b = (0.2 * rng.standard_normal(64)).astype(np.float16)
    emb = (rng.standard_normal((37, 64)) * 0.5).astype(np.float16)
    got = O.lm_head_logits(cfg, x, g, b, emb)
    assert got.dtype == np.float32 and got.shape == (5, 37)
    y = torch.nn.functional.layer_norm(torch.from_numpy(x.astype(np.float64)), (64,),
                                       torch.from_numpy(g.astype(np.float64)), torch.from_numpy(b.astype(np.float64)),
                                       cfg.ln_eps)
    y = y.to(torch.float16).to(torch.float64)                               # FP16 storage of the LN output
    ref = (y @ torch.from_numpy(emb.astype(np.float64)).T).numpy()
    assert np.allclose(got, ref, rtol=2e-6, atol=2e-6)
    # the pieces that must be there: without the LN, or with the untransposed / another matrix, it differs
    no_ln = x.astype(np.float64) @ emb.astype(np.float64).T
    assert np.abs(got - no_ln).max() > 0.5


def test_lm_head_one_hot_state_selects_one_embedding_column():
    """Closed form.  With gamma = 1, beta = 0 a hidden state c*e_j normalises to
    (e_j - 1/h) * c / sqrt(c^2 (1/h)(1 - 1/h) + eps); its logit against embedding row v is therefore
    a * (E[v, j] - mean(E[v, :])): the head reads COLUMN j of E (row-major [vocab, h1], tied), which
    pins orientation and tying, and the centring pins the final LayerNorm."""
    h, vocab, j, c = 64, 23, 17, 4.0
    rng = np.random.default_rng(5)
    emb = (rng.standard_normal((vocab, h))).astype(np.float16)
    cfg = O.ModelCfg(h1=h, nh=1, h2=128, vocab=vocab, max_pos=8)
    x = np.zeros((1, h), np.float16)
    x[0, j] = c
    got = O.lm_head_logits(cfg, x, np.ones(h, np.float16), np.zeros(h, np.float16), emb)[0].astype(np.float64)
    var = c * c * (1.0 / h) * (1.0 - 1.0 / h)
    inv = 1.0 / np.sqrt(var + cfg.ln_eps)
    y = np.full(h, -c / h * inv)
    y[j] = (c - c / h) * inv
    y = y.astype(np.float16).astype(np.float64)                              # FP16 storage of the LN output
    ref = np.array([sum(float(y[k]) * float(emb[v, k]) for k in range(h)) for v in range(vocab)])
    assert np.allclose(got, ref, rtol=1e-6, atol=1e-6)
    # ... which is, up to the FP16 rounding of y, a multiple of the centred column j of E
    e64 = emb.astype(np.float64)
    approx = (c * inv) * (e64[:, j] - e64.mean(axis=1))
    assert np.abs(got - approx).max() < 2e-2 * np.abs(approx).max()
    assert int(O.greedy(got[None].astype(np.float32))[0]) == int(np.argmax(e64[:, j] - e64.mean(axis=1)))


def test_generate_first_token_from_independent_pieces():
    """Token 1 of generate() recomputed with torch float64 for the model-level glue (embedding sum,
    final LayerNorm, tied head) around the oracle's own prefill_layer (pinned in test_oracle_layer)."""
    import torch
    sh, cfg, layers, m = _tiny_model(quant=True)
    prompt = synth.prompt_ids(2, 6, sh.vocab, 2)
    ids = O.generate(cfg, layers, m["embed"], m["pos"], m["lnf_g"], m["lnf_b"], prompt, 1, 1, 2, True)
    E = torch.from_numpy(m["embed"].astype(np.float64))
    P = torch.from_numpy(m["pos"].astype(np.float64))
    x = (E[torch.from_numpy(prompt.astype(np.int64))] + P[:6][None]).to(torch.float16).numpy()
    for j in range(2):
        x = O.prefill_layer(cfg, layers[j], x, O.KVCache.empty(2, sh.nh, 7, sh.dh, True))
    y = torch.nn.functional.layer_norm(torch.from_numpy(x[:, -1].astype(np.float64)), (sh.h1,),
                                       torch.from_numpy(m["lnf_g"].astype(np.float64)),
                                       torch.from_numpy(m["lnf_b"].astype(np.float64)), cfg.ln_eps)
    logits = (y.to(torch.float16).to(torch.float64) @ E.T).to(torch.float32)
    assert np.array_equal(ids[:, 0], torch.argmax(logits, dim=-1).numpy().astype(np.int32))
