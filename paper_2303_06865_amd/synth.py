"""Seeded synthetic inputs shared by the tests, the smoke check and the benchmark.

Holds no arithmetic of the method: only random draws with the shapes and value
distributions of the paper's throughput workload (Section 6: equal-length
prompts, dummy weights).  Each tensor gets its own stream derived from
(seed, layer, tensor id), so any single layer can be regenerated alone.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, Optional

import numpy as np

# tensor ids for per-tensor seeding
T_WQKV, T_WO, T_W1, T_W2, T_BQKV, T_BO, T_B1, T_B2, T_LN1G, T_LN1B, T_LN2G, T_LN2B = range(12)
T_EMBED, T_POS, T_LNFG, T_LNFB, T_PROMPT, T_X, T_Q, T_K, T_V = range(100, 109)


@dataclass(frozen=True)
class Shape:
    """Model shape in the paper's notation: h1 hidden, nh heads, h2 FFN hidden."""
    h1: int
    nh: int
    h2: int
    vocab: int
    max_pos: int
    l: int = 1
    ln_eps: float = 1e-5

    @property
    def dh(self) -> int:
        return self.h1 // self.nh


OPT_125M_LAYER = Shape(h1=768, nh=12, h2=3072, vocab=50272, max_pos=2048, l=1)
OPT_6_7B = Shape(h1=4096, nh=32, h2=16384, vocab=50272, max_pos=2048, l=32)
OPT_30B = Shape(h1=7168, nh=56, h2=28672, vocab=50272, max_pos=2048, l=48)
OPT_175B = Shape(h1=12288, nh=96, h2=49152, vocab=50272, max_pos=2048, l=96)


def rng(seed: int, layer: int, tensor_id: int) -> np.random.Generator:
    return np.random.default_rng([int(seed), int(layer) + 1, int(tensor_id)])


def normal_f16(shape, std: float, seed: int, layer: int, tensor_id: int) -> np.ndarray:
    g = rng(seed, layer, tensor_id)
    return (g.standard_normal(shape, dtype=np.float32) * np.float32(std)).astype(np.float16)


def layer_tensors(sh: Shape, seed: int, layer: int, std: float = 0.02, biases: bool = False,
                  random_ln: bool = False) -> Dict[str, Optional[np.ndarray]]:
    """FP16 tensors of one decoder layer: weights ~ N(0, std), LayerNorm gamma=1,
    beta=0 (or mildly random when random_ln), biases absent (or ~ N(0, std))."""
    h1, h2 = sh.h1, sh.h2
    t: Dict[str, Optional[np.ndarray]] = {
        "wqkv": normal_f16((3 * h1, h1), std, seed, layer, T_WQKV),
        "wo": normal_f16((h1, h1), std, seed, layer, T_WO),
        "w1": normal_f16((h2, h1), std, seed, layer, T_W1),
        "w2": normal_f16((h1, h2), std, seed, layer, T_W2),
    }
    if biases:
        t["bqkv"] = normal_f16((3 * h1,), std, seed, layer, T_BQKV)
        t["bo"] = normal_f16((h1,), std, seed, layer, T_BO)
        t["b1"] = normal_f16((h2,), std, seed, layer, T_B1)
        t["b2"] = normal_f16((h1,), std, seed, layer, T_B2)
    else:
        t["bqkv"] = t["bo"] = t["b1"] = t["b2"] = None
    if random_ln:
        t["ln1_g"] = (1.0 + normal_f16((h1,), 0.1, seed, layer, T_LN1G).astype(np.float32)).astype(np.float16)
        t["ln1_b"] = normal_f16((h1,), 0.1, seed, layer, T_LN1B)
        t["ln2_g"] = (1.0 + normal_f16((h1,), 0.1, seed, layer, T_LN2G).astype(np.float32)).astype(np.float16)
        t["ln2_b"] = normal_f16((h1,), 0.1, seed, layer, T_LN2B)
    else:
        t["ln1_g"] = np.ones(h1, np.float16)
        t["ln1_b"] = np.zeros(h1, np.float16)
        t["ln2_g"] = np.ones(h1, np.float16)
        t["ln2_b"] = np.zeros(h1, np.float16)
    return t


def model_tensors(sh: Shape, seed: int, std: float = 0.02) -> Dict[str, np.ndarray]:
    """Token embedding (tied LM head), learned positions, final LayerNorm."""
    return {
        "embed": normal_f16((sh.vocab, sh.h1), std, seed, -1, T_EMBED),
        "pos": normal_f16((sh.max_pos, sh.h1), std, seed, -1, T_POS),
        "lnf_g": np.ones(sh.h1, np.float16),
        "lnf_b": np.zeros(sh.h1, np.float16),
    }


def prompt_ids(bls: int, s: int, vocab: int, seed: int) -> np.ndarray:
    """Equal-length prompts of uniform random token ids (Section 6 workload)."""
    return rng(seed, -1, T_PROMPT).integers(0, vocab, size=(bls, s), dtype=np.int32)


def activations_f16(shape, std: float, seed: int, tensor_id: int = T_X) -> np.ndarray:
    return normal_f16(shape, std, seed, -1, tensor_id)
