"""End-to-end parity of fg_generate (block schedule, Algorithm 1) against the oracle: greedy token
ids must be identical; where a GPU id differs, the test fails unless the oracle's own top-2 logit
margin at that step is below the measured logit error (reported, never hidden)."""
import numpy as np
import pytest
import torch

from oracle import fg_oracle as O
from paper_2303_06865_amd import binding as B
from paper_2303_06865_amd import synth
from tests.util import cfg_pair, dev, host, oracle_layer

pytestmark = pytest.mark.gpu


def _models(sh, seed, quant, std, biases, random_ln):
    ocfg, cfg = cfg_pair(sh)
    olayers, layers = [], []
    for j in range(sh.l):
        t = synth.layer_tensors(sh, seed, j, std=std, biases=biases, random_ln=random_ln)
        olayers.append(oracle_layer(t, quant))
        layers.append(B.LayerWeights.from_numpy(t, quant))
    m = synth.model_tensors(sh, seed, std=std)
    return ocfg, cfg, olayers, layers, m


def _gpu_generate(cfg, layers, m, prompt, n, ngb, gbs, quant_kv):
    bls, s = prompt.shape
    kv = [B.KVCache(cfg, bls, s + n, quant_kv) for _ in layers]
    ids, stats = B.fg_generate(cfg, layers, dev(m["embed"]), dev(m["pos"]), dev(m["lnf_g"]), dev(m["lnf_b"]),
                               dev(prompt), n, ngb, gbs, kv)
    torch.cuda.synchronize()
    return host(ids), stats


def _compare_ids(got, ref, logits, err=2e-3):
    """Ids must be equal.  The one admissible exception is a near-tie: the GPU's token is the
    oracle's runner-up region, i.e. the oracle's own logit gap between its winner and the GPU's
    choice is below 4 x `err` x rms of that logit row, `err` being the relative logit error to
    expect: 2e-3 with FP16 caches; 1e-2 with 4-bit caches, where the two sides' caches differ by
    whole quantization steps in a fraction of a percent of their entries (an FP16 ulp of difference
    in a K/V value that crosses a rounding boundary) and short contexts average little of that
    away.  Such events are printed; a sequence is not compared past its first near-tie because its
    later tokens legitimately follow a different prefix.  Returns the number of near-ties."""
    ties = 0
    for b, i in np.argwhere(got != ref):
        if np.any(got[b, :i] != ref[b, :i]):
            continue
        row = logits[i, b].astype(np.float64)
        gap = float(row[ref[b, i]] - row[got[b, i]])
        allowed = 4 * err * float(np.sqrt((row ** 2).mean()))
        assert 0 <= gap < allowed, "sequence %d step %d: ids %d vs %d, oracle gap %.3e (near-tie bound %.3e)" % (
            b, i, got[b, i], ref[b, i], gap, allowed)
        print("near-tie: sequence %d step %d ids %d vs %d, oracle gap %.3e < %.3e" % (
            b, i, got[b, i], ref[b, i], gap, allowed))
        ties += 1
    return ties


@pytest.mark.parametrize("n", [9, 8])
def test_generate_opt125m_config(n):
    """OPT-125m-shaped single layer, batch 4, prompt 32, seed 0: n = 9 gives 8 decode steps after
    the prefill token, n = 8 is the other reading of '8 greedy decode steps'."""
    sh = synth.OPT_125M_LAYER
    ocfg, cfg, olayers, layers, m = _models(sh, 0, True, 0.02, False, False)
    prompt = synth.prompt_ids(4, 32, sh.vocab, 0)
    ref, logits, _ = O.generate(ocfg, olayers, m["embed"], m["pos"], m["lnf_g"], m["lnf_b"], prompt, n, 1, 4, True,
                                return_trace=True)
    got, stats = _gpu_generate(cfg, layers, m, prompt, n, 1, 4, True)
    assert got.shape == (4, n)
    _compare_ids(got, ref, logits)
    assert np.array_equal(got, ref)
    assert stats["tokens"] == 4 * n and stats["prefill_s"] > 0 and len(stats["decode_step_s"]) == n - 1
    w_elems = 4 * 768 * 768 + 2 * 768 * 3072
    assert stats["weight_bytes_per_step"] == w_elems * 5 // 8
    assert stats["kv_bytes_last_step"] == 2 * 4 * 768 * (32 + n - 1) * 5 // 8


@pytest.mark.parametrize("quant", [True, False])
def test_generate_small_multilayer_and_factorisations(quant):
    """Three layers, biases, random LayerNorm parameters; the ids must not depend on how the block
    of 6 sequences is cut into GPU batches (sequences of a block are independent)."""
    sh = synth.Shape(h1=256, nh=4, h2=512, vocab=2000, max_pos=64, l=3)
    ocfg, cfg, olayers, layers, m = _models(sh, 7, quant, 0.08, True, True)
    prompt = synth.prompt_ids(6, 11, sh.vocab, 7)
    ref, logits, _ = O.generate(ocfg, olayers, m["embed"], m["pos"], m["lnf_g"], m["lnf_b"], prompt, 6, 2, 3, quant,
                                return_trace=True)
    outs = []
    for ngb, gbs in ((1, 6), (2, 3), (6, 1), (3, 2)):
        got, _ = _gpu_generate(cfg, layers, m, prompt, 6, ngb, gbs, quant)
        assert _compare_ids(got, ref, logits, 1e-2 if quant else 2e-3) <= 1
        outs.append(got)
    for o in outs[1:]:
        assert np.array_equal(o, outs[0])


def test_generate_single_token_and_async_call():
    """n = 1 is prefill only; stats = NULL leaves the call fully asynchronous."""
    sh = synth.Shape(h1=128, nh=2, h2=256, vocab=520, max_pos=32, l=2)
    ocfg, cfg, olayers, layers, m = _models(sh, 9, True, 0.08, True, True)
    prompt = synth.prompt_ids(3, 5, sh.vocab, 9)
    ref = O.generate(ocfg, olayers, m["embed"], m["pos"], m["lnf_g"], m["lnf_b"], prompt, 1, 1, 3, True)
    kv = [B.KVCache(cfg, 3, 8, True) for _ in layers]
    ids, stats = B.fg_generate(cfg, layers, dev(m["embed"]), dev(m["pos"]), dev(m["lnf_g"]), dev(m["lnf_b"]),
                               dev(prompt), 1, 1, 3, kv, want_stats=False)
    torch.cuda.synchronize()
    assert stats is None and np.array_equal(host(ids), ref)


# ------------------------------------------------------------------ diagonal block schedule
@pytest.mark.parametrize("n_seqs,gbs,s,n,meta_f16", [
    (6, 2, 11, 6, False),     # fewer batches than steps: all in flight together
    (8, 1, 9, 3, False),      # more batches than steps: pages are recycled
    (4, 2, 60, 7, True),      # sequences grow across a page boundary; FP16-pair pages
    (3, 3, 5, 1, False),      # n = 1: prefill iterations only
])
def test_generate_diagonal_schedule(n_seqs, gbs, s, n, meta_f16):
    """Appendix, diagonal block schedule over paged caches: the ids are those of the oracle's block
    schedule (the oracle pins its own diagonal order to it), the page peak is the oracle's."""
    sh = synth.Shape(h1=256, nh=4, h2=512, vocab=2000, max_pos=96, l=3)
    ocfg, cfg, olayers, layers, m = _models(sh, 11, True, 0.08, True, True)
    prompt = synth.prompt_ids(n_seqs, s, sh.vocab, 13)
    ref, logits, _ = O.generate(ocfg, olayers, m["embed"], m["pos"], m["lnf_g"], m["lnf_b"], prompt, n, n_seqs // gbs,
                                gbs, True, return_trace=True)
    _, opeak = O.generate_diagonal(ocfg, olayers[:1], m["embed"], m["pos"], m["lnf_g"], m["lnf_b"], prompt, n, gbs,
                                   return_page_use=True)
    need = B.fg_diagonal_pages_needed(n_seqs, s, n, gbs)
    assert need == opeak
    pages = [B.KVPages(cfg, need, meta_f16, zero=False) for _ in layers]
    for p in pages:     # the pool's previous contents must not matter
        p.k_codes.random_(0, 256)
        p.v_codes.random_(0, 256)
    ids, st = B.fg_generate_diagonal(cfg, layers, dev(m["embed"]), dev(m["pos"]), dev(m["lnf_g"]), dev(m["lnf_b"]),
                                     dev(prompt), n, gbs, pages)
    torch.cuda.synchronize()
    got = host(ids)
    assert got.shape == (n_seqs, n) and st["tokens"] == n_seqs * n and st["peak_pages"] == need and st["total_s"] > 0
    assert _compare_ids(got, ref, logits, 1e-2) <= 1


def test_generate_diagonal_rejects_a_pool_that_is_too_small():
    sh = synth.Shape(h1=128, nh=2, h2=256, vocab=520, max_pos=96, l=1)
    ocfg, cfg, olayers, layers, m = _models(sh, 9, True, 0.08, True, True)
    prompt = synth.prompt_ids(4, 70, sh.vocab, 9)
    need = B.fg_diagonal_pages_needed(4, 70, 4, 1)
    assert need == 8 and B.fg_diagonal_pages_needed(4, 70, 4, 3) == -1
    pages = [B.KVPages(cfg, need - 1)]
    with pytest.raises(RuntimeError):
        B.fg_generate_diagonal(cfg, layers, dev(m["embed"]), dev(m["pos"]), dev(m["lnf_g"]), dev(m["lnf_b"]),
                               dev(prompt), 4, 1, pages)
