"""The five synthetic workloads and the rule that fixes each one's training-state shard.

Sizes only: a hidden width, a head count, an MLP width, a sequence length, a
batch share b = l * m, a precision mode and a shard rule.  The number of flat
parameters P is supplied by the caller (the oracle and the HIP library each
count it with their own layout code), so no layout arithmetic lives here.
"""
from dataclasses import dataclass
import numpy as np


@dataclass(frozen=True)
class LayerConfig:
    name: str
    hidden: int          # H
    heads: int           # A
    mlp: int             # F
    seq: int             # S
    causal: bool
    micro_batch: int     # m, samples per micro-batch
    n_micro: int         # l, micro-batches in this GPU's share (b = l * m)
    dtype: str           # "f32" or "bf16" (bf16 operands, fp32 master/grad/accumulate)
    layers: int = 1      # > 1: a full stack with embedding and LM head
    vocab: int = 0
    seed: int = 0
    lr: float = 1e-3
    shard_rule: str = ""
    kind: str = "gpt"    # "gpt": LayerNorm, biases, GELU; "llama": RMSNorm, rotary embedding, gated SiLU, no biases
    init_std: float = 0.02   # standard deviation of the weight matrices' draws

    @property
    def batch_share(self):
        return self.micro_batch * self.n_micro

    @property
    def tokens_per_micro(self):
        return self.micro_batch * self.seq

    @property
    def tokens_per_step(self):
        return self.batch_share * self.seq


CONFIGS = {
    # tiny GPT-style layer, fp32
    "c1": LayerConfig("c1", 256, 4, 1024, 128, True, 2, 2, "f32", seed=1001, shard_rule="frac:37:41"),
    # BERT-large-shaped layer (sizes only), non-causal
    "c2": LayerConfig("c2", 1024, 16, 4096, 512, False, 2, 4, "bf16", seed=1002, shard_rule="frac:50:23"),
    # GPT-2-XL-shaped layer
    "c3": LayerConfig("c3", 1600, 25, 6400, 1024, True, 2, 3, "bf16", seed=1003, shard_rule="split4"),
    # 7B-class layer
    "c4": LayerConfig("c4", 4096, 32, 16384, 2048, True, 1, 4, "bf16", seed=1004, shard_rule="third_odd"),
    # full 24-layer GPT stack with tied embedding
    "c5": LayerConfig("c5", 2048, 16, 8192, 2048, True, 2, 6, "bf16", layers=24, vocab=50257, seed=1005,
                      shard_rule="frac29_seeded"),
    # Llama-style layers (sizes only): a 7B-class layer (H 4096, 32 heads, F 11008) and a small one for the oracle
    "l7b": LayerConfig("l7b", 4096, 32, 11008, 2048, True, 1, 4, "bf16", seed=1006, shard_rule="third_odd", kind="llama"),
    # TinyLlama-shaped stack (the paper's model table: 22 layers, H 2048, 32 heads; F 5632 and a 32000-entry vocabulary
    # are that model family's): the Llama-style counterpart of c5
    "ltiny": LayerConfig("ltiny", 2048, 32, 5632, 2048, True, 2, 6, "bf16", layers=22, vocab=32000, seed=1008,
                         shard_rule="frac29_seeded", kind="llama"),
    "lstackmini": LayerConfig("lstackmini", 256, 4, 688, 136, True, 2, 2, "bf16", layers=2, vocab=1031, seed=1108,
                              shard_rule="frac:37:41", kind="llama"),
    "lmini": LayerConfig("lmini", 256, 4, 688, 136, True, 2, 2, "bf16", seed=1106, shard_rule="frac:37:41", kind="llama"),
    # ViT-Large-shaped encoder layer: 197 tokens per image, non-causal (the GPT-style layer form)
    "vitl": LayerConfig("vitl", 1024, 16, 4096, 197, False, 8, 2, "bf16", seed=1007, shard_rule="frac:50:23"),
    # two more of the paper's model table whose head widths are neither 64 nor 128: a GPT 2.7B-shaped layer (80 heads
    # of 32) and a ViT-G-shaped one (16 heads of 104, 257 tokens per image)
    "g27": LayerConfig("g27", 2560, 80, 10240, 2048, True, 1, 4, "bf16", seed=1009, shard_rule="third_odd"),
    "vitg": LayerConfig("vitg", 1664, 16, 8192, 257, False, 8, 2, "bf16", seed=1010, shard_rule="frac:50:23"),
    # reduced relatives used only by parity tests (ragged tiles, small enough for the oracle)
    "c5mini": LayerConfig("c5mini", 256, 4, 1024, 128, True, 2, 2, "bf16", layers=2, vocab=1031, seed=1105,
                          shard_rule="frac29_seeded"),
}


def get_config(name):
    return CONFIGS[name]


def split4_boundaries(P, seed):
    """Boundaries e_0..e_4 of a seeded uneven 4-way split of [0, P)."""
    rng = np.random.Generator(np.random.Philox(key=seed + 77))
    w = rng.uniform(0.5, 1.5, size=4)
    c = np.concatenate([[0.0], np.cumsum(w)]) / np.sum(w)
    e = [int(np.floor(P * ck)) for ck in c]
    e[0], e[4] = 0, P
    return e


def shard_of(cfg, P):
    """(offset, length) of this GPU's slice of the P flat training-state elements."""
    rule = cfg.shard_rule
    if rule.startswith("frac:"):
        _, fo, fl = rule.split(":")
        return (P * int(fo)) // 100, (P * int(fl)) // 100
    if rule == "split4":
        e = split4_boundaries(P, cfg.seed)
        k = cfg.seed % 4
        return e[k], e[k + 1] - e[k]
    if rule == "third_odd":
        ln = P // 3
        off = ln if ln % 2 == 1 else ln + 1
        return off, ln
    if rule == "frac29_seeded":
        ln = (P * 29) // 100
        rng = np.random.Generator(np.random.Philox(key=cfg.seed + 78))
        off = int(np.floor(rng.uniform() * (P - ln)))
        return off, ln
    raise ValueError(rule)
