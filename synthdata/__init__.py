"""Seeded synthetic inputs: model shapes, weights, sequence lengths, token batches.

This module is the only code that both the CPU oracle's tests and the HIP
library's tests/bench use.  It holds none of the method's arithmetic: it only
names tensor shapes and draws random numbers.  Everything is generated from one
64-bit seed with numpy's PCG64 so both sides receive byte-identical arrays.

The workloads stand in for the fine-tuning batches of the paper's evaluation
(Section 3.1: sequence lengths 35-141, 153-512 and 30-332 for the three
datasets, "normal / power-law like" distributions; Section 6.1, Table 1:
batch sizes 12-32), which are not available here.  Every batch has one
sequence length L shared by all of its B samples (the paper pads to the longest
sample of the batch, Section 2.1), token ids are uniform over the vocabulary and
weights are N(0, 0.02).
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field, asdict
from typing import Dict, List, Tuple

import numpy as np

MASTER_SEED = 220902478


@dataclass(frozen=True)
class ModelShape:
    n_layers: int
    hidden: int
    n_heads: int
    ffn: int
    vocab: int
    max_seq: int
    dtype: str = "fp32"        # "fp32" | "bf16" (bf16 storage, fp32 accumulation)
    causal: int = 0            # 1: causal decoder
    pre_ln: int = 0            # 1: pre-LN blocks + final LN
    gelu_tanh: int = 0         # 1: tanh approximation of GELU
    head: int = 1              # 1: MLM head (dense+GELU+LN, tied decoder + bias); 0: tied LM head only
    ln_eps: float = 1e-5
    ffn_by_layer: Tuple[int, ...] = ()   # stacks whose layers differ: feed-forward width per layer (empty: ffn)

    def ffn_of(self, l: int) -> int:
        return self.ffn_by_layer[l] if self.ffn_by_layer else self.ffn


@dataclass(frozen=True)
class Workload:
    name: str
    shape: ModelShape
    batch: int
    length_recipe: Tuple          # see seq_lengths()
    steps: int
    budget_frac: float            # budget = frac * (no-checkpoint peak at L = max_seq)
    seed: int


WORKLOADS: Dict[str, Workload] = {
    "tiny": Workload(
        "tiny", ModelShape(2, 64, 2, 256, 1000, 64, "fp32"),
        4, ("uniform_int", 16, 64, 1), 20, 0.70, MASTER_SEED + 0),
    "bert_base": Workload(
        "bert_base", ModelShape(12, 768, 12, 3072, 30522, 512, "bf16"),
        32, ("lognormal", 200.0, 0.5, 64, 512, 8), 200, 0.60, MASTER_SEED + 1),
    "bert_large": Workload(
        "bert_large", ModelShape(24, 1024, 16, 4096, 30522, 512, "bf16"),
        64, ("uniform_int", 128, 512, 16), 100, 0.50, MASTER_SEED + 2),
    "gpt2_medium": Workload(
        "gpt2_medium", ModelShape(24, 1024, 16, 4096, 50257, 1024, "bf16",
                                  causal=1, pre_ln=1, gelu_tanh=1, head=0),
        16, ("lognormal", 400.0, 0.6, 128, 1024, 1), 100, 0.45, MASTER_SEED + 3),
    "bert_large_stress": Workload(
        "bert_large_stress", ModelShape(24, 1024, 16, 4096, 30522, 512, "bf16"),
        256, ("bimodal", 32, 96, 384, 512, 8), 500, 0.30, MASTER_SEED + 4),
    # stacks whose layers differ (the stages of Section 4.4): three stages with feed-forward
    # widths stepping down, so that the layers fall into three buckets of Algorithm 1; the mean
    # width, and with it the work per token, is that of bert_base
    "tiny_stages": Workload(
        "tiny_stages", ModelShape(4, 64, 2, 256, 1000, 64, "fp32", ffn_by_layer=(512, 512, 128, 128)),
        4, ("uniform_int", 16, 64, 1), 24, 0.70, MASTER_SEED + 5),
    "bert_stages": Workload(
        "bert_stages", ModelShape(12, 768, 12, 3072, 30522, 512, "bf16",
                                  ffn_by_layer=(4096,) * 4 + (3072,) * 4 + (2048,) * 4),
        32, ("lognormal", 200.0, 0.5, 64, 512, 8), 200, 0.60, MASTER_SEED + 6),
}


def shape_dict(shape: ModelShape) -> dict:
    return asdict(shape)


def param_shapes(s: ModelShape) -> List[Tuple[str, Tuple[int, ...], str]]:
    """Canonical list of (name, shape, kind); kind in {"normal","zeros","ones"}.

    Linear weights are stored [out_features, in_features]; the fused QKV weight
    stacks the query, key and value projections along the output axis.
    """
    H, V = s.hidden, s.vocab
    out: List[Tuple[str, Tuple[int, ...], str]] = [
        ("tok_emb", (V, H), "normal"),
        ("pos_emb", (s.max_seq, H), "normal"),
    ]
    if not s.pre_ln:
        out += [("emb_ln_g", (H,), "ones"), ("emb_ln_b", (H,), "zeros")]
    for l in range(s.n_layers):
        p = f"layer{l}."
        F = s.ffn_of(l)
        out += [
            (p + "wqkv", (3 * H, H), "normal"), (p + "bqkv", (3 * H,), "zeros"),
            (p + "wo", (H, H), "normal"), (p + "bo", (H,), "zeros"),
            (p + "ln1_g", (H,), "ones"), (p + "ln1_b", (H,), "zeros"),
            (p + "w1", (F, H), "normal"), (p + "b1", (F,), "zeros"),
            (p + "w2", (H, F), "normal"), (p + "b2", (H,), "zeros"),
            (p + "ln2_g", (H,), "ones"), (p + "ln2_b", (H,), "zeros"),
        ]
    if s.pre_ln:
        out += [("final_ln_g", (H,), "ones"), ("final_ln_b", (H,), "zeros")]
    if s.head:
        out += [
            ("head.wt", (H, H), "normal"), ("head.bt", (H,), "zeros"),
            ("head.ln_g", (H,), "ones"), ("head.ln_b", (H,), "zeros"),
            ("head.bdec", (V,), "zeros"),
        ]
    return out


def make_params(s: ModelShape, seed: int, perturb: bool = False) -> Dict[str, np.ndarray]:
    """fp32 parameters.  Default init: weights N(0, 0.02), biases 0, LN (1, 0).

    With perturb=True biases and LN parameters also receive small random values,
    so that parity tests exercise every term (a zero bias hides a wrong bias path).
    """
    rng = np.random.Generator(np.random.PCG64(seed))
    params: Dict[str, np.ndarray] = {}
    for name, shp, kind in param_shapes(s):
        if kind == "normal":
            a = rng.standard_normal(shp, dtype=np.float64) * 0.02
        elif kind == "ones":
            a = np.ones(shp)
            if perturb:
                a = a + 0.1 * rng.standard_normal(shp)
        else:
            a = np.zeros(shp)
            if perturb:
                a = a + 0.05 * rng.standard_normal(shp)
        params[name] = a.astype(np.float32)
    return params


def seq_lengths(recipe: Tuple, steps: int, seed: int) -> List[int]:
    """Per-step sequence length L, drawn once per step."""
    rng = np.random.Generator(np.random.PCG64(seed ^ 0x5EC1E7))
    kind = recipe[0]
    out: List[int] = []
    if kind == "uniform_int":
        _, lo, hi, step = recipe
        choices = list(range(lo, hi + 1, step))
        out = [int(choices[i]) for i in rng.integers(0, len(choices), size=steps)]
    elif kind == "lognormal":
        _, median, sigma, lo, hi, rnd = recipe
        z = rng.standard_normal(steps)
        raw = np.exp(math.log(median) + sigma * z)
        raw = np.clip(raw, lo, hi)
        out = [int(min(hi, max(lo, rnd * int(round(v / rnd))))) for v in raw]
    elif kind == "bimodal":
        _, lo1, hi1, lo2, hi2, step = recipe
        c1 = list(range(lo1, hi1 + 1, step))
        c2 = list(range(lo2, hi2 + 1, step))
        coin = rng.integers(0, 2, size=steps)
        i1 = rng.integers(0, len(c1), size=steps)
        i2 = rng.integers(0, len(c2), size=steps)
        out = [int(c1[a]) if c == 0 else int(c2[b]) for c, a, b in zip(coin, i1, i2)]
    else:
        raise ValueError(f"unknown length recipe {kind!r}")
    return out


def make_batch(s: ModelShape, B: int, L: int, seed: int) -> Tuple[np.ndarray, np.ndarray]:
    """tokens[B, L] and labels[B, L] (int32).

    Encoder shapes: labels are independent uniform ids at every position.
    Causal shapes: the label of position p is the token at p+1 and the last
    position carries no label (-1).
    """
    rng = np.random.Generator(np.random.PCG64(seed))
    tokens = rng.integers(0, s.vocab, size=(B, L), dtype=np.int64).astype(np.int32)
    if s.causal:
        labels = np.full((B, L), -1, dtype=np.int32)
        labels[:, :-1] = tokens[:, 1:]
    else:
        labels = rng.integers(0, s.vocab, size=(B, L), dtype=np.int64).astype(np.int32)
    return tokens, labels


def make_padded_batch(s: ModelShape, lengths, seed: int) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """tokens[B, L], labels[B, L], lengths[B] (int32) of a batch whose samples have their own
    lengths and are padded to the longest, L = max(lengths).

    Padding positions hold token id 0 and label -1.  Causal shapes: the last real token of a
    sample has no successor and carries no label.
    """
    lengths = np.asarray(lengths, dtype=np.int32)
    B, L = len(lengths), int(lengths.max())
    tokens, labels = make_batch(s, B, L, seed)
    for b, n in enumerate(lengths):
        tokens[b, n:] = 0
        labels[b, n:] = -1
        if s.causal:
            labels[b, n - 1] = -1
    return tokens, labels, lengths


def step_seed(workload_seed: int, step: int) -> int:
    return (workload_seed * 1000003 + step * 7919 + 17) & 0x7FFFFFFFFFFFFFFF
