"""GPU-vs-oracle parity protocol, shared by the GPU tests, smoke() and nothing else.

The GPU free-runs greedy decoding through the C ABI; the oracle is
teacher-forced on the ids the GPU emitted and produces float64 logits for the
same history.  Logits must agree within `tol`; the GPU id must equal the
oracle's argmax unless the oracle's top-2 margin is below `margin`.
"""
from __future__ import annotations

import numpy as np


def gpu_generate(model, prompts_np, n_new, want_logits=True):
    """Run prefill + n_new decode steps.  Returns (ids [B, n_new], logits [B, n_new, V] or None)."""
    import torch
    with model.on_stream():          # the model's own stream is torch's current one: no waits between calls
        toks = torch.from_numpy(np.ascontiguousarray(prompts_np, dtype=np.int32)).to(model.device)
        model.bt_prefill(toks)
        ids, lgs = [], []
        for _ in range(n_new):
            ids.append(model.bt_decode_step().clone())
            if want_logits:
                lgs.append(model.bt_get_logits())
        ids = torch.stack(ids, 1)
        lgs = torch.stack(lgs, 1) if want_logits else None
    torch.cuda.synchronize()
    return ids.cpu().numpy(), (lgs.cpu().numpy() if want_logits else None)


def compare_with_oracle(cfg, weights, prompts_np, gpu_ids, gpu_logits, tol, margin=2e-2, seqs=None):
    """Teacher-force the cached oracle on gpu_ids; returns a report dict and asserts nothing."""
    import oracle.block_transformer as O
    sel = list(range(prompts_np.shape[0])) if seqs is None else list(seqs)
    P = O.Params(weights)
    n_new = gpu_ids.shape[1]
    _, o_logits, _ = O.generate_cached(P, cfg, prompts_np[sel], n_new, forced=gpu_ids[sel])
    diff = np.abs(gpu_logits[sel].astype(np.float64) - o_logits)
    srt = np.sort(o_logits, axis=-1)
    o_margin = srt[..., -1] - srt[..., -2] if o_logits.shape[-1] > 1 else np.full(o_logits.shape[:2], np.inf)
    o_ids = np.argmax(o_logits, axis=-1)
    mism = gpu_ids[sel] != o_ids
    return {
        "max_abs_logit_diff": float(diff.max()),
        "steps": int(mism.size),
        "exempt_mismatches": int(np.sum(mism & (o_margin < margin))),
        "true_mismatches": int(np.sum(mism & (o_margin >= margin))),
        "tol": tol,
    }


def gpu_generate_ragged(model, prompts, n_new):
    """prompts: list of 1-D id arrays of different lengths.  Returns (ids [B, n_new], logits [B, n_new, V])."""
    import torch
    lens = [len(p) for p in prompts]
    buf = np.full((len(prompts), max(lens)), 1, dtype=np.int32)      # the tail of a shorter row must not be read
    for b, p in enumerate(prompts):
        buf[b, :lens[b]] = p
    with model.on_stream():
        model.bt_prefill_ragged(torch.from_numpy(buf).to(model.device), lens)
        ids, lgs = [], []
        for _ in range(n_new):
            ids.append(model.bt_decode_step().clone())
            lgs.append(model.bt_get_logits())
        ids, lgs = torch.stack(ids, 1), torch.stack(lgs, 1)
    torch.cuda.synchronize()
    return ids.cpu().numpy(), lgs.cpu().numpy()


def compare_ragged_with_oracle(cfg, weights, prompts, gpu_ids, gpu_logits, tol, margin=2e-2):
    """As compare_with_oracle for a batch of prompts of different lengths."""
    import oracle.block_transformer as O
    _, o_logits = O.generate_ragged(O.Params(weights), cfg, prompts, gpu_ids.shape[1], forced=gpu_ids)
    diff = np.abs(gpu_logits.astype(np.float64) - o_logits)
    srt = np.sort(o_logits, axis=-1)
    o_margin = srt[..., -1] - srt[..., -2]
    mism = gpu_ids != np.argmax(o_logits, axis=-1)
    return {
        "max_abs_logit_diff": float(diff.max()),
        "steps": int(mism.size),
        "exempt_mismatches": int(np.sum(mism & (o_margin < margin))),
        "true_mismatches": int(np.sum(mism & (o_margin >= margin))),
        "tol": tol,
    }


def assert_parity(rep):
    assert rep["max_abs_logit_diff"] <= rep["tol"], rep
    assert rep["true_mismatches"] == 0, rep


# ---------------------------------------------------------------------------
# full-size workloads: sampled steps of sampled sequences
# ---------------------------------------------------------------------------
def gpu_generate_sampled(model, prompts_np, n_new, seqs, steps):
    """Full-batch generation; logits are kept only for `seqs` at decode steps `steps`.

    Returns (ids [B, n_new] int32, {step: float32 [len(seqs), V]}).
    """
    import torch
    want = set(int(s) for s in steps)
    kept = {}
    with model.on_stream():
        toks = torch.from_numpy(np.ascontiguousarray(prompts_np, dtype=np.int32)).to(model.device)
        sel = torch.tensor(list(seqs), device=model.device, dtype=torch.long)
        ids = torch.empty(n_new, prompts_np.shape[0], dtype=torch.int32, device=model.device)
        model.bt_prefill(toks)
        for t in range(n_new):
            model.bt_decode_step(ids[t])
            if t in want:
                kept[t] = model.bt_get_logits()[sel].clone()
    torch.cuda.synchronize()
    return ids.t().contiguous().cpu().numpy(), {t: v.cpu().numpy() for t, v in kept.items()}


def sample_steps(cfg, n_new):
    """First two blocks, one block in the middle, the last complete block."""
    L = cfg.block_len
    st = set(range(min(2 * L, n_new)))
    mid = (n_new // 2) // L * L
    st |= set(range(mid, min(mid + L, n_new)))
    last = (n_new - 1) // L * L
    st |= set(range(last, n_new))
    return sorted(st)


def compare_sampled_with_oracle(cfg, weights, prompts_np, gpu_ids, gpu_logits, seqs, tol, margin=2e-2):
    """Oracle logits (plain definition, teacher-forced on the GPU's history) at the sampled steps."""
    import oracle.block_transformer as O
    seqs = list(seqs)
    L = cfg.block_len
    P = O.Params(weights, keep=False)
    padded = O.left_pad(cfg, prompts_np[seqs])           # no-op for whole blocks
    T_p = padded.shape[1]
    hist = np.concatenate([padded, gpu_ids[seqs]], axis=1).astype(np.int64)
    steps = sorted(gpu_logits)
    blocks = sorted({(T_p + t) // L for t in steps})
    tf = O.teacher_forced_logits(P, cfg, hist, blocks)
    worst, exempt, true_mm = 0.0, 0, 0
    for t in steps:
        i, k = (T_p + t) // L, (T_p + t) % L
        ref = tf[i][:, k]
        dmax = float(np.max(np.abs(gpu_logits[t].astype(np.float64) - ref)))
        worst = max(worst, dmax) if np.isfinite(dmax) else float("inf")      # a NaN logit fails the tolerance
        srt = np.sort(ref, axis=-1)
        o_margin = srt[:, -1] - srt[:, -2]
        mism = gpu_ids[seqs, t] != np.argmax(ref, axis=-1)
        exempt += int(np.sum(mism & (o_margin < margin)))
        true_mm += int(np.sum(mism & (o_margin >= margin)))
    return {"max_abs_logit_diff": worst, "steps": len(steps) * len(seqs), "exempt_mismatches": exempt,
            "true_mismatches": true_mm, "tol": tol}
