"""Seeded synthetic inputs for the Block Transformer generation step.

This module serves both the CPU oracle and the HIP path and holds none of the
method's arithmetic: only the workload table (shapes), the weight generator
and the prompt generator.  Everything is deterministic in its seeds.

The paper trains on the Pile with a 50 304-entry vocabulary and times inference
on synthetic prompts padded to the target length (Appendix E, settings for
Section 3.2).  Neither the corpus nor trained weights exist here, so prompts
are drawn from a Zipf law (a stand-in for natural token frequency) and weights
from N(0, 0.02^2).

Tensor layouts (shared by both sides):
  * every linear map is stored [out_features, in_features], row-major, and is
    applied as y = x @ W.T + b;
  * W_qkv rows are ordered q (D rows), k (D rows), v (D rows); inside each
    part head h owns rows [h*d_h, (h+1)*d_h);
  * W_prefix is [P*D, D]; prefix token p is output slice [p*D, (p+1)*D).
In bf16 mode the matrices and embedding tables are held as raw bf16 bit
patterns (uint16, round-to-nearest-even from the fp32 draw); biases and
LayerNorm parameters stay fp32.
"""
from __future__ import annotations

import os
import threading
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, replace
from typing import Dict

import numpy as np

__all__ = [
    "BTConfig", "CONFIGS", "get_config", "make_weights", "make_prompts",
    "f32_to_bf16_bits", "bf16_bits_to_f32", "MATRIX_NAMES", "LAYER_TENSORS",
]


@dataclass(frozen=True)
class BTConfig:
    name: str
    dtype: str              # "fp32" or "bf16"
    vocab: int
    block_len: int          # L_B
    d_model: int            # D (both decoders)
    n_heads: int
    d_ff: int
    n_block_layers: int
    n_token_layers: int
    prefix_len: int         # P (0 only with block_len == 1)
    batch: int
    prompt_len: int
    gen_len: int
    prompt_dist: str        # "uniform" or "zipf"
    weights_seed: int
    prompt_seed: int
    rotary_dims: int = -1   # per head; -1 -> d_head // 4
    parallel_residual: int = 1
    ln_eps: float = 1e-5
    pad_id: int = 0         # fills the first block of a prompt whose length is not a multiple of L_B
    eos_id: int = -1        # -1: none; else a sequence that emitted it keeps emitting it
    token_mix: str = "prefix"   # how the context embedding enters the token decoder: "prefix" or "sum"

    @property
    def d_emb(self) -> int:
        return self.d_model // self.block_len

    @property
    def d_head(self) -> int:
        return self.d_model // self.n_heads

    @property
    def rot(self) -> int:
        return self.d_head // 4 if self.rotary_dims < 0 else self.rotary_dims

    @property
    def n_prompt_blocks(self) -> int:
        return -(-self.prompt_len // self.block_len)

    @property
    def max_blocks(self) -> int:
        return self.n_prompt_blocks + self.gen_len // self.block_len

    @property
    def n_prefix_rows(self) -> int:
        """Rows the token decoder sees for the context embedding."""
        return max(self.prefix_len, 1)

    @property
    def n_proj(self) -> int:
        """Vectors of dimension D the context embedding is projected to: prefix_len prefix tokens, or
        block_len summands (token_mix == "sum"); W_prefix is [n_proj * D, D]."""
        return self.block_len if self.token_mix == "sum" else self.prefix_len

    def with_(self, **kw) -> "BTConfig":
        return replace(self, **kw)


def _cfg(idx, name, dtype, vocab, lb, d, h, f, nb, nt, p, batch, tp, tg, dist):
    return BTConfig(name=name, dtype=dtype, vocab=vocab, block_len=lb, d_model=d,
                    n_heads=h, d_ff=f, n_block_layers=nb, n_token_layers=nt,
                    prefix_len=p, batch=batch, prompt_len=tp, gen_len=tg,
                    prompt_dist=dist, weights_seed=1000 + idx, prompt_seed=2000 + idx)


# The five workloads plus the vanilla-equivalent comparison run of the last one.
CONFIGS: Dict[str, BTConfig] = {
    "cfg0": _cfg(0, "cfg0", "fp32", 512, 4, 128, 4, 512, 2, 2, 1, 2, 32, 32, "uniform"),
    "cfg1": _cfg(1, "cfg1", "bf16", 50304, 4, 768, 12, 3072, 12, 12, 1, 64, 128, 2048, "zipf"),
    "cfg2": _cfg(2, "cfg2", "bf16", 50304, 4, 768, 12, 3072, 12, 12, 1, 32, 2048, 128, "zipf"),
    "cfg3": _cfg(3, "cfg3", "bf16", 50304, 8, 1024, 16, 4096, 16, 16, 2, 128, 128, 2048, "zipf"),
    "cfg4": _cfg(4, "cfg4", "bf16", 50304, 4, 2048, 16, 8192, 24, 24, 1, 256, 2048, 2048, "zipf"),
    "cfg4v": _cfg(4, "cfg4v", "bf16", 50304, 1, 2048, 16, 8192, 24, 24, 0, 256, 2048, 2048, "zipf"),
}


def get_config(name: str) -> BTConfig:
    return CONFIGS[name]


# ----------------------------------------------------------------------------
# bf16 bit helpers (storage format only: 1 sign, 8 exponent, 7 mantissa bits)
# ----------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to the nearest bf16 (ties to even); returns uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = u + (np.uint32(0x7FFF) + lsb)
    return (r >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns to the fp32 values they denote (exact)."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


# ----------------------------------------------------------------------------
# Weights
# ----------------------------------------------------------------------------
# (name, kind) per transformer layer, in generation order.  kind: "mat" (stored
# in the model dtype), "vec" (fp32 bias / LN beta), "gamma" (fp32, 1 + noise).
LAYER_TENSORS = (
    ("ln1_g", "gamma"), ("ln1_b", "vec"),
    ("W_qkv", "mat"), ("b_qkv", "vec"),
    ("W_o", "mat"), ("b_o", "vec"),
    ("ln2_g", "gamma"), ("ln2_b", "vec"),
    ("W_up", "mat"), ("b_up", "vec"),
    ("W_down", "mat"), ("b_down", "vec"),
)
MATRIX_NAMES = ("E_emb", "E_tok", "W_prefix", "W_head", "W_qkv", "W_o", "W_up", "W_down")


def _layer_shapes(cfg: BTConfig):
    D, F = cfg.d_model, cfg.d_ff
    return {
        "ln1_g": (D,), "ln1_b": (D,), "W_qkv": (3 * D, D), "b_qkv": (3 * D,),
        "W_o": (D, D), "b_o": (D,), "ln2_g": (D,), "ln2_b": (D,),
        "W_up": (F, D), "b_up": (F,), "W_down": (D, F), "b_down": (D,),
    }


def tensor_table(cfg: BTConfig):
    """Ordered list of (name, shape, kind) for every tensor of the model."""
    D, V, P = cfg.d_model, cfg.vocab, cfg.n_proj
    out = [("E_emb", (V, cfg.d_emb), "mat"), ("E_tok", (V, D), "mat")]
    if P > 0:
        out += [("W_prefix", (P * D, D), "mat"), ("b_prefix", (P * D,), "vec")]
    out += [("W_head", (V, D), "mat"),
            ("blk_lnf_g", (D,), "gamma"), ("blk_lnf_b", (D,), "vec"),
            ("tok_lnf_g", (D,), "gamma"), ("tok_lnf_b", (D,), "vec")]
    shapes = _layer_shapes(cfg)
    for stack, n in (("blk", cfg.n_block_layers), ("tok", cfg.n_token_layers)):
        for i in range(n):
            for nm, kind in LAYER_TENSORS:
                out.append((f"{stack}.{i}.{nm}", shapes[nm], kind))
    return out


def make_weights(cfg: BTConfig, std: float = 0.02) -> Dict[str, np.ndarray]:
    """All tensors of the model, each from its own child stream of weights_seed.

    Matrices ~ N(0, std^2); biases and LN beta ~ N(0, std^2) so that every code
    path is exercised; LN gamma = 1 + N(0, std^2).  fp32 mode: float32 arrays.
    bf16 mode: matrices are uint16 bf16 bit patterns, vectors float32.

    Large tensors are drawn piece by piece into one reused buffer (the generator's stream does not
    depend on how a draw is cut up, so the values are those of a single draw): the billions of
    weights of the large workloads would otherwise spend most of their time in page faults of
    temporaries.
    """
    table = tensor_table(cfg)
    children = np.random.SeedSequence(cfg.weights_seed).spawn(len(table))
    piece = 1 << 22
    local = threading.local()

    def one(item):
        (name, shape, kind), ss = item
        if not hasattr(local, "buf"):
            local.buf = np.empty(piece, dtype=np.float32)
            local.tmp = np.empty(piece, dtype=np.uint32)
        rng = np.random.Generator(np.random.PCG64(ss))
        n = int(np.prod(shape))
        to_bf16 = kind == "mat" and cfg.dtype == "bf16"
        res = np.empty(n, dtype=np.uint16 if to_bf16 else np.float32)
        for i in range(0, n, piece):
            m = min(piece, n - i)
            w = local.buf[:m]
            rng.standard_normal(m, dtype=np.float32, out=w)
            w *= np.float32(std)
            if kind == "gamma":
                w += np.float32(1.0)
            if to_bf16:
                # round to nearest even, as f32_to_bf16_bits does, without temporaries
                u = w.view(np.uint32)
                t = local.tmp[:m]
                np.right_shift(u, np.uint32(16), out=t)
                t &= np.uint32(1)
                t += np.uint32(0x7FFF)
                t += u
                t >>= np.uint32(16)
                res[i:i + m] = t
            else:
                res[i:i + m] = w
        return name, res.reshape(shape)

    # every tensor has its own stream, so the tensors can be drawn side by side (numpy releases the
    # interpreter lock inside the generator and the element-wise passes)
    workers = max(1, min(8, os.cpu_count() or 1))
    with ThreadPoolExecutor(max_workers=workers) as ex:
        return dict(ex.map(one, zip(table, children)))


# ----------------------------------------------------------------------------
# Prompts
# ----------------------------------------------------------------------------
def make_prompts(cfg: BTConfig, batch: int | None = None, prompt_len: int | None = None) -> np.ndarray:
    """int32 [batch, prompt_len] token ids.

    "uniform": uniform over [0, vocab).  "zipf": rank k in 1..V with
    p(k) proportional to k^-1.1, id = k-1, drawn by inverse CDF.
    """
    B = cfg.batch if batch is None else batch
    T = cfg.prompt_len if prompt_len is None else prompt_len
    rng = np.random.default_rng(cfg.prompt_seed)
    if cfg.prompt_dist == "uniform":
        return rng.integers(0, cfg.vocab, size=(B, T), dtype=np.int64).astype(np.int32)
    if cfg.prompt_dist == "zipf":
        k = np.arange(1, cfg.vocab + 1, dtype=np.float64)
        cdf = np.cumsum(k ** -1.1)
        cdf /= cdf[-1]
        u = rng.random(size=(B, T))
        ids = np.searchsorted(cdf, u, side="left")
        return np.minimum(ids, cfg.vocab - 1).astype(np.int32)
    raise ValueError(cfg.prompt_dist)
