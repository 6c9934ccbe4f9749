"""Parity at the workloads' full sizes, in the launch configuration bench.py times.

The GPU runs the whole batch; the oracle (plain definition, teacher-forced on
the ids the GPU emitted) checks sampled decode steps of sampled sequences:
the first and the last of the batch, which are independent of the others.
"""
import time

import numpy as np
import pytest

from parity import assert_parity, compare_sampled_with_oracle, gpu_generate_sampled, sample_steps
from synth import CONFIGS, make_prompts, make_weights

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def amd():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    import paper_2406_02657_amd as amd
    return amd


def full_size_case(amd, cfg, n_new, seqs, batch=None, prompt_len=None, also_without_logits=False):
    t0 = time.time()
    W = make_weights(cfg)
    prompts = make_prompts(cfg, batch=batch, prompt_len=prompt_len)
    B, T = prompts.shape
    print(f"[{cfg.name}] inputs {time.time() - t0:.1f}s", flush=True)
    m = amd.Model(cfg, W, max_batch=B, max_blocks=(T + n_new) // cfg.block_len + 1)
    steps = sample_steps(cfg, n_new)
    t0 = time.time()
    ids, lgs = gpu_generate_sampled(m, prompts, n_new, seqs, steps)
    st = m.bt_get_stats()
    m.close()
    print(f"[{cfg.name}] gpu {time.time() - t0:.1f}s  B={B} T_p={T} n_new={n_new}", flush=True)
    assert st.graph_fallback == 0 and st.graph_launches > n_new - 3 * (cfg.block_len + 1)     # the steps ran as graph replays
    if also_without_logits:
        # the configuration bench.py times: the LM head leaves argmax candidates only (keep_logits = 0)
        m = amd.Model(cfg, W, max_batch=B, max_blocks=(T + n_new) // cfg.block_len + 1, keep_logits=0)
        ids0, _ = gpu_generate_sampled(m, prompts, n_new, seqs, [])
        m.close()
        assert np.array_equal(ids0, ids)
    assert ids.min() >= 0 and ids.max() < cfg.vocab
    n_p = -(-T // cfg.block_len)
    assert st.block_passes == n_p + -(-n_new // cfg.block_len) - 1
    assert st.token_passes == n_new
    t0 = time.time()
    rep = compare_sampled_with_oracle(cfg, W, prompts, ids, lgs, seqs, 2e-2)
    print(f"[{cfg.name}] oracle {time.time() - t0:.1f}s {rep}", flush=True)
    assert_parity(rep)


def test_cfg1_decode_heavy_full(amd):
    cfg = CONFIGS["cfg1"]
    full_size_case(amd, cfg, cfg.gen_len, [0, cfg.batch - 1], also_without_logits=True)


def test_cfg2_prefill_heavy_full(amd):
    cfg = CONFIGS["cfg2"]
    full_size_case(amd, cfg, cfg.gen_len, [0, cfg.batch - 1], also_without_logits=True)


def test_cfg3_medium_full(amd):
    cfg = CONFIGS["cfg3"]
    full_size_case(amd, cfg, cfg.gen_len, [0, cfg.batch - 1])


def test_cfg4_large(amd):
    """Full batch, full prompt, all 2048 decode steps (the cache grows from 512 to 1023 blocks at
    d_head = 128); one sequence, sampled steps: the first two blocks, a middle block, the last block."""
    cfg = CONFIGS["cfg4"]
    full_size_case(amd, cfg, cfg.gen_len, [cfg.batch - 1])


def test_cfg4v_vanilla_equivalent(amd):
    """L_B = 1, no prefix, at cfg4's width, depth, batch and prompt length (one KV entry per token):
    the first 256 decode steps, one sequence, sampled steps.  The cache is sized for these steps
    (2305 entries per sequence, 116 GB); the full 4096 are what bench.py --workload cfg4v times."""
    cfg = CONFIGS["cfg4v"]
    full_size_case(amd, cfg, 256, [cfg.batch - 1])


def test_cfg4v_small_batch_every_kind_of_step(amd):
    """The same model at batch 8 with 512-token prompts: a second sequence position and cache length."""
    cfg = CONFIGS["cfg4v"]
    full_size_case(amd, cfg, 64, [7], batch=8, prompt_len=512)


def test_cfg1_model_long_context(amd):
    """8K-token prompts on cfg1's model (the long-context setting of the paper's appendix on
    context lengths): 2048 cached blocks per sequence after prefill."""
    cfg = CONFIGS["cfg1"]
    full_size_case(amd, cfg, 24, [0, 15], batch=16, prompt_len=8192)


def test_cfg1_model_unaligned_no_prompt(amd):
    """Full batch, one-token prompts (the setting without an input sequence): L_B - 1 pads."""
    cfg = CONFIGS["cfg1"]
    full_size_case(amd, cfg, 64, [0, cfg.batch - 1], prompt_len=1)


def test_cfg1_model_scoring(amd):
    """bt_score on cfg1's model: 16 sequences of 2176 tokens (cfg1's prompt + generation length), the
    workspace's default row budget (several prefill chunks), checked on three blocks of two sequences."""
    import oracle.block_transformer as O
    import torch
    cfg = CONFIGS["cfg1"]
    T = cfg.prompt_len + cfg.gen_len
    W = make_weights(cfg)
    toks = make_prompts(cfg, batch=16, prompt_len=T)
    m = amd.Model(cfg, W, max_batch=16, max_blocks=T // cfg.block_len, score_rows=4096)
    nll = m.bt_score(torch.from_numpy(toks).to(m.device)).cpu().numpy()
    m.close()
    assert np.isfinite(nll).all() and np.all(nll[:, :cfg.block_len] == 0) and np.all(nll[:, cfg.block_len:] > 0)
    seqs, blocks = [0, 15], [1, 271, T // cfg.block_len - 1]
    lg = O.teacher_forced_logits(O.Params(W, keep=False), cfg, toks[seqs].astype(np.int64), blocks)
    L = cfg.block_len
    for i in blocks:
        z = lg[i]
        lse = z.max(axis=-1) + np.log(np.exp(z - z.max(axis=-1, keepdims=True)).sum(axis=-1))
        want = lse - np.take_along_axis(z, toks[seqs, i * L:(i + 1) * L].astype(np.int64)[..., None], axis=-1)[..., 0]
        got = nll[seqs, i * L:(i + 1) * L]
        print(f"[cfg1 scoring] block {i}: max |d nll| {np.abs(got - want).max():.2e}", flush=True)
        assert np.abs(got - want).max() <= 4e-2
