"""bt_create_static: the entry point for callers that cannot allocate device memory.

A model whose workspace is the library's static device array must give what a model on a
caller-allocated workspace gives: same kernels, same launches, so ids and logits are compared
bit for bit (and the static model's output once more against the oracle, at the usual tolerance).
Two calls in a row, the second with a smaller model, batch and cache: the array still holds the
first model's contents then.
"""
import numpy as np
import pytest

from helpers import tiny_cfg
from parity import assert_parity, compare_with_oracle, gpu_generate
from synth import make_prompts, make_weights

pytestmark = pytest.mark.gpu


def test_static_workspace_model_equals_bt_create():
    import torch
    assert torch.cuda.is_available(), "this test needs the MI355X"
    import paper_2406_02657_amd as amd
    big = tiny_cfg(dtype="bf16", d_model=256, n_heads=4, d_ff=512, vocab=700, block_len=4, prefix_len=2, prompt_len=24)
    small = tiny_cfg(dtype="bf16", d_model=128, n_heads=2, d_ff=256, vocab=300, block_len=4, prefix_len=1, prompt_len=9,
                     weights_seed=8)
    for cfg, batch, n_new, blocks in ((big, 6, 21, 40), (small, 2, 10, 8)):
        W = make_weights(cfg)
        prompts = make_prompts(cfg, batch=batch)
        ref = amd.Model(cfg, W, max_batch=batch, max_blocks=blocks, use_graphs=0)
        want = gpu_generate(ref, prompts, n_new)
        ref.close()
        m = amd.Model(cfg, W, max_batch=batch, max_blocks=blocks, static_workspace=True)
        assert m.workspace is None and m.workspace_bytes <= 32 << 20
        # a second live model on the same static array is refused
        h2 = amd.binding._P()
        assert amd.lib.bt_create_static(amd.binding.C.byref(m.c), amd.binding.C.byref(m.w), None,
                                        amd.binding.C.byref(h2)) == amd.binding.BT_ERR_STATE
        got = gpu_generate(m, prompts, n_new)
        got2 = gpu_generate(m, prompts, n_new)          # re-entrant on the same array
        st = m.bt_get_stats()
        m.close()
        assert st.graph_launches == 0 and st.graph_captures == 0
        assert np.array_equal(want[0], got[0]) and np.array_equal(want[1], got[1])
        assert np.array_equal(want[0], got2[0]) and np.array_equal(want[1], got2[1])
        assert_parity(compare_with_oracle(cfg, W, prompts, got[0], got[1], 2e-2))
