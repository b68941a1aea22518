"""Seeded, synthetic stand-ins for the paper's generation workload.

The paper generates long-form reasoning traces with a Qwen-2.5-shaped 7B policy at a
constant batch per GPU, refilling finished sequences and swapping weights in flight
(Alg. 2; experimental setup in Sec. 5).  Neither its prompts nor its checkpoints are
used here: every weight, prompt, length and KV value below is drawn from a seeded
generator with the same shapes and length mix.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
import numpy as np

__all__ = [
    "ModelCfg", "CONFIGS", "weight_names", "weight_shapes", "make_weights", "perturb_weights",
    "bf16_round", "f32_to_bf16_bits", "bf16_bits_to_f32", "random_prompts", "lognormal_lengths",
    "stationary_ages", "attention_microbench_lengths",
]


@dataclass(frozen=True)
class ModelCfg:
    """Decoder shape (pre-norm RMSNorm, RoPE, grouped-query attention, SwiGLU, untied LM head)."""
    n_layers: int
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    d_ffn: int
    vocab: int
    rope_theta: float = 1.0e4
    rms_eps: float = 1.0e-6

    @property
    def q_dim(self) -> int:
        return self.n_q_heads * self.head_dim

    @property
    def kv_dim(self) -> int:
        return self.n_kv_heads * self.head_dim

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    def kv_bytes_per_token(self) -> int:
        return 2 * self.n_layers * self.n_kv_heads * self.head_dim * 2

    def streamed_params(self) -> int:
        """Weights every decode step has to read: all layers, final norm, LM head."""
        d, f = self.d_model, self.d_ffn
        per_layer = 2 * d + (self.q_dim + 2 * self.kv_dim) * d + d * self.q_dim + 2 * f * d + d * f
        return self.n_layers * per_layer + d + self.vocab * d

    def with_layers(self, n: int) -> "ModelCfg":
        return replace(self, n_layers=n)


# The five workload shapes of the benchmark description (tiny, 1.5B, attention-only, 7B, 32B).
CONFIGS = {
    "tiny": ModelCfg(2, 256, 8, 2, 32, 1024, 4096),
    "1p5b": ModelCfg(28, 1536, 12, 2, 128, 8960, 151936),
    "attn": ModelCfg(1, 3584, 28, 4, 128, 18944, 152064),
    "7b": ModelCfg(28, 3584, 28, 4, 128, 18944, 152064),
    "32b": ModelCfg(64, 5120, 40, 8, 128, 27648, 152064),
}


def weight_names(cfg: ModelCfg) -> list[str]:
    names = ["embed"]
    for l in range(cfg.n_layers):
        names += [f"l{l}.g1", f"l{l}.wq", f"l{l}.wk", f"l{l}.wv", f"l{l}.wo",
                  f"l{l}.g2", f"l{l}.wg", f"l{l}.wu", f"l{l}.wd"]
    names += ["gf", "lm_head"]
    return names


def weight_shapes(cfg: ModelCfg) -> dict[str, tuple[int, ...]]:
    """Every projection is stored [out_features, in_features]; y = x @ W.T."""
    d, f = cfg.d_model, cfg.d_ffn
    shp: dict[str, tuple[int, ...]] = {"embed": (cfg.vocab, d)}
    for l in range(cfg.n_layers):
        shp[f"l{l}.g1"] = (d,)
        shp[f"l{l}.wq"] = (cfg.q_dim, d)
        shp[f"l{l}.wk"] = (cfg.kv_dim, d)
        shp[f"l{l}.wv"] = (cfg.kv_dim, d)
        shp[f"l{l}.wo"] = (d, cfg.q_dim)
        shp[f"l{l}.g2"] = (d,)
        shp[f"l{l}.wg"] = (f, d)
        shp[f"l{l}.wu"] = (f, d)
        shp[f"l{l}.wd"] = (d, f)
    shp["gf"] = (d,)
    shp["lm_head"] = (cfg.vocab, d)
    return shp


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even fp32 -> bf16, returned as uint16 bit patterns (finite inputs)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def bf16_round(x: np.ndarray) -> np.ndarray:
    """The fp32 value of x after storage in bf16."""
    return bf16_bits_to_f32(f32_to_bf16_bits(x)).reshape(np.shape(x))


def make_weights(cfg: ModelCfg, seed: int, std: float = 0.02) -> dict[str, np.ndarray]:
    """fp32 master weights: matrices ~ N(0, std^2), norm gains = 1."""
    rng = np.random.default_rng(seed)
    out = {}
    for name, shp in weight_shapes(cfg).items():
        if len(shp) == 1:
            out[name] = np.ones(shp, dtype=np.float32)
        else:
            out[name] = (rng.standard_normal(shp, dtype=np.float32) * np.float32(std))
    return out


def perturb_weights(master: dict[str, np.ndarray], seed: int, std: float = 1.0e-3) -> dict[str, np.ndarray]:
    """The 'next optimizer step' stand-in: W' = W + N(0, std^2) on every tensor, gains included."""
    rng = np.random.default_rng(seed)
    return {k: (v + rng.standard_normal(v.shape, dtype=np.float32) * np.float32(std)).astype(np.float32)
            for k, v in master.items()}


def random_prompts(rng: np.random.Generator, n: int, length: int, vocab: int) -> np.ndarray:
    return rng.integers(0, vocab, size=(n, length), dtype=np.int32)


def lognormal_lengths(rng: np.random.Generator, n: int, mean: float, lo: int, hi: int,
                      sigma: float = 0.75) -> np.ndarray:
    """clip(round(exp(N(mu, sigma^2))), lo, hi) with mu chosen so the unclipped mean is `mean`."""
    mu = np.log(mean) - 0.5 * sigma * sigma
    g = np.rint(np.exp(rng.normal(mu, sigma, size=n)))
    return np.clip(g, lo, hi).astype(np.int64)


def stationary_ages(rng: np.random.Generator, n: int, mean: float, lo: int, hi: int,
                    sigma: float = 0.75, pool: int = 200_000) -> tuple[np.ndarray, np.ndarray]:
    """Generation length G and tokens already generated (age) of the sequences found in flight
    once constant-batch refill has reached steady state: G is length-biased (a slot is busy
    with a long sequence for longer), the age is uniform in [0, G)."""
    cand = lognormal_lengths(rng, pool, mean, lo, hi, sigma)
    p = cand / cand.sum()
    g = rng.choice(cand, size=n, p=p)
    age = np.floor(rng.random(n) * g).astype(np.int64)
    return g.astype(np.int64), age


def attention_microbench_lengths(seed: int, batch: int = 512, mean: float = 4096.0,
                                 lo: int = 128, hi: int = 16384) -> np.ndarray:
    return lognormal_lengths(np.random.default_rng(seed), batch, mean, lo, hi)
