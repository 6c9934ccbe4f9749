"""Shared test helpers: tiny model configs (shapes only, no arithmetic)."""
from synth import BTConfig


def tiny_cfg(**kw):
    base = dict(name="tiny", dtype="fp32", vocab=37, block_len=4, d_model=32, n_heads=4,
                d_ff=64, n_block_layers=2, n_token_layers=2, prefix_len=2, batch=2,
                prompt_len=8, gen_len=9, prompt_dist="uniform", weights_seed=7,
                prompt_seed=11, rotary_dims=-1, parallel_residual=1, ln_eps=1e-5)
    base.update(kw)
    return BTConfig(**base)
