"""The five benchmark configurations (grammar, vocabulary, batch, steps, logits dtype)."""
from dataclasses import dataclass
from . import grammars, vocab
from .rng import MASTER_SEED, stream


@dataclass(frozen=True)
class Config:
    index: int
    name: str
    V: int
    batch: int
    steps: int
    dtype: str      # "f32" | "bf16"
    sigma: float

    @property
    def seed(self) -> int:
        return MASTER_SEED + self.index

    def grammar(self):
        if self.index in (1, 2):
            return grammars.json_grammar()
        if self.index == 3:
            return grammars.json_schema_grammar(self.seed)
        if self.index == 4:
            return grammars.semantic_grammar(self.seed)
        return grammars.expr_grammar()

    def vocab(self, size=None):
        return vocab.make_vocab(self.seed, size or self.V, uniform_2_8=(self.index == 1),
                                non_ascii=(self.index != 1))

    def sampler(self, row: int):
        return stream(self.seed, f"sample[{row}]")


CONFIGS = {
    1: Config(1, "json_v2k", 2048, 1, 64, "f32", 1.0),
    2: Config(2, "json_v32k", 32000, 1, 256, "f32", 1.0),
    3: Config(3, "json_schema_v128k", 128256, 16, 512, "bf16", 2.0),
    4: Config(4, "semantic_v128k", 128256, 64, 256, "bf16", 2.0),
    5: Config(5, "expr_v152k", 152064, 64, 1024, "f32", 1.0),
}


def pick_set_bit(mask_words, r: int) -> int:
    """Index of the r-th (0-based) set bit of a little-endian-bit uint32 word array."""
    for w, word in enumerate(mask_words):
        word = int(word)
        c = bin(word).count("1")
        if r < c:
            for b in range(32):
                if (word >> b) & 1:
                    if r == 0:
                        return w * 32 + b
                    r -= 1
        r -= c
    raise IndexError("r exceeds popcount")


def make_logits(cfg: Config, step: int, device="cpu", batch=None, V=None):
    """Seeded N(0, sigma) logits [batch, V] in the configuration's dtype (torch tensor)."""
    import torch
    g = torch.Generator(device="cpu")
    g.manual_seed((cfg.seed * 1000003 + step) & 0x7FFFFFFFFFFFFFFF)
    x = torch.randn((batch or cfg.batch, V or cfg.V), generator=g, dtype=torch.float32) * cfg.sigma
    if cfg.dtype == "bf16":
        x = x.to(torch.bfloat16)
    return x.to(device)
