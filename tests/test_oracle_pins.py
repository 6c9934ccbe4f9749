"""Pins for the CPU oracle: things the paper and the mathematics fix.

Each test is chosen so that a plausible mistake in the oracle (a dropped term,
a wrong mask bound, a transposed operand, a position off by one) fails it.
Citations are to arXiv 2406.02657.
"""
import math
import os

import numpy as np
import pytest

import oracle.block_transformer as O
from synth import CONFIGS, make_prompts, make_weights, tensor_table
from helpers import tiny_cfg

TOL = 1e-10


def build(cfg):
    return O.Params(make_weights(cfg))


# --------------------------------------------------------------------------
# T1  cached mode == full recomputation (Sec. 2.1; Fig. 1; App. C)
# --------------------------------------------------------------------------
@pytest.mark.parametrize("lb,p", [(1, 1), (2, 1), (4, 2), (8, 3), (4, 1), (1, 0)])
@pytest.mark.parametrize("parallel", [1, 0])
@pytest.mark.parametrize("rot", [-1, 0])
def test_cached_equals_full(lb, p, parallel, rot):
    cfg = tiny_cfg(block_len=lb, prefix_len=p, parallel_residual=parallel, rotary_dims=rot,
                   prompt_len=2 * lb, d_model=32, n_heads=2)
    P = build(cfg)
    prompts = make_prompts(cfg, batch=3)
    n_new = 2 * lb + 3
    ids_f, lg_f = O.generate_full(P, cfg, prompts, n_new)
    ids_c, lg_c, _ = O.generate_cached(P, cfg, prompts, n_new)
    assert np.array_equal(ids_f, ids_c)
    assert np.max(np.abs(lg_f - lg_c)) < TOL


def test_teacher_forced_equals_stepwise():
    cfg = tiny_cfg(block_len=4, prefix_len=2)
    P = build(cfg)
    rng = np.random.default_rng(0)
    toks = rng.integers(0, cfg.vocab, size=(2, 20))
    tf = O.teacher_forced_logits(P, cfg, toks, [1, 3, 4])
    for i in (1, 3, 4):
        for k in range(cfg.block_len):
            t = i * cfg.block_len + k
            ref = O.next_token_logits_full(P, cfg, toks[:, :t])
            assert np.max(np.abs(tf[i][:, k] - ref)) < TOL
    # and the cached generator forced onto the same history
    _, lg_c, _ = O.generate_cached(P, cfg, toks[:, :8], 12, forced=toks[:, 8:])
    for t in range(8, 20):
        ref = O.next_token_logits_full(P, cfg, toks[:, :t])
        assert np.max(np.abs(lg_c[:, t - 8] - ref)) < TOL


# --------------------------------------------------------------------------
# T2  locality of the token decoder, causality of the block decoder
#     (Sec. 2.4: each block is processed independently; Sec. 2.3)
# --------------------------------------------------------------------------
def test_token_decoder_locality_bit_identical():
    cfg = tiny_cfg(block_len=4, prefix_len=2)
    P = build(cfg)
    rng = np.random.default_rng(1)
    c = rng.standard_normal((2, cfg.d_model))
    blk = rng.integers(0, cfg.vocab, size=(2, 3))
    base = O.block_logits(P, cfg, c, blk)
    # block_logits has no other input: anything outside (c, current block) cannot matter.
    # Same check through the cached generator: hold the context fixed, vary history.
    toks_a = rng.integers(0, cfg.vocab, size=(2, 12))
    toks_b = toks_a.copy()
    toks_b[:, :8] = rng.integers(0, cfg.vocab, size=(2, 8))      # different earlier blocks
    outs = []
    for toks in (toks_a, toks_b):
        g = O.CachedGenerator(P, cfg, 2, 8)
        g.prefill(toks[:, :8])
        g.c = c.copy()                                             # inject the context
        lg = [g.step(forced_ids=toks[:, 8 + k])[0] for k in range(4)]
        outs.append(np.stack(lg, 1))
    assert np.array_equal(outs[0], outs[1])                        # bit-identical
    # a token inside the current block does matter
    blk2 = blk.copy()
    blk2[:, 0] = (blk2[:, 0] + 1) % cfg.vocab
    other = O.block_logits(P, cfg, c, blk2)
    assert np.array_equal(other[:, 0], base[:, 0])                 # before the edit: same
    assert np.max(np.abs(other[:, 1:] - base[:, 1:])) > 1e-6       # after it: different


def test_block_decoder_causality():
    cfg = tiny_cfg(block_len=2, prefix_len=1)
    P = build(cfg)
    rng = np.random.default_rng(2)
    toks = rng.integers(0, cfg.vocab, size=(1, 12))
    base = O.context_embeddings(P, cfg, toks)
    for j in range(6):
        t2 = toks.copy()
        t2[0, 2 * j] = (t2[0, 2 * j] + 1) % cfg.vocab
        out = O.context_embeddings(P, cfg, t2)
        assert np.array_equal(out[:, :j], base[:, :j])             # earlier outputs untouched
        assert np.all(np.max(np.abs(out[:, j:] - base[:, j:]), axis=-1) > 1e-9)  # later all change


# --------------------------------------------------------------------------
# T3  L_B = 1 reduces to a vanilla transformer (Sec. 3.5 "Analysis on vanilla
#     ... to block": L_B=1 differs from vanilla only by local attention in the
#     upper layers).  The vanilla model below shares no code with the oracle.
# --------------------------------------------------------------------------
def _v_ln(x, g, b, eps):
    mu = sum(x) / len(x)
    var = sum((xi - mu) ** 2 for xi in x) / len(x)
    return np.array([(xi - mu) / math.sqrt(var + eps) for xi in x]) * g + b


def _v_gelu(u):
    return np.array([0.5 * ui * (1.0 + math.erf(ui / math.sqrt(2.0))) for ui in u])


def _v_rot(vec, pos, rot):
    out = vec.copy()
    for t in range(rot // 2):
        th = pos * (10000.0 ** (-2.0 * t / rot))
        a, b = vec[t], vec[t + rot // 2]
        out[t] = a * math.cos(th) - b * math.sin(th)
        out[t + rot // 2] = b * math.cos(th) + a * math.sin(th)
    return out


def vanilla_forward(W, x_rows, layers, H, rot, eps, parallel):
    """Textbook decoder stack on one sequence.  x_rows: [T, D] input embeddings.

    layers: list of (prefix, mask) where mask[i][j] says whether position i may
    attend to position j, or ("ln", gname, bname) for a LayerNorm stage.
    Written with per-position, per-head Python loops on purpose.
    """
    f = lambda nm: np.asarray(W[nm], dtype=np.float64)
    T, D = x_rows.shape
    dh = D // H
    x = [x_rows[t].astype(np.float64) for t in range(T)]
    for st in layers:
        if st[0] == "ln":
            x = [_v_ln(xt, f(st[1]), f(st[2]), eps) for xt in x]
            continue
        pre, mask, positions = st

        def attn(inp):
            q, k, v = [], [], []
            for t in range(T):
                u = _v_ln(inp[t], f(pre + "ln1_g"), f(pre + "ln1_b"), eps)
                z = f(pre + "W_qkv") @ u + f(pre + "b_qkv")
                q.append(z[:D]); k.append(z[D:2 * D]); v.append(z[2 * D:])
            out = []
            for t in range(T):
                o = np.zeros(D)
                for h in range(H):
                    sl = slice(h * dh, (h + 1) * dh)
                    qt = _v_rot(q[t][sl], positions[t], rot)
                    js = [j for j in range(T) if mask[t][j]]
                    sc = [float(qt @ _v_rot(k[j][sl], positions[j], rot)) / math.sqrt(dh) for j in js]
                    m = max(sc)
                    e = [math.exp(s - m) for s in sc]
                    z = sum(e)
                    for w8, j in zip(e, js):
                        o[sl] += (w8 / z) * v[j][sl]
                out.append(f(pre + "W_o") @ o + f(pre + "b_o"))
            return out

        def mlp(inp):
            out = []
            for t in range(T):
                u = _v_ln(inp[t], f(pre + "ln2_g"), f(pre + "ln2_b"), eps)
                out.append(f(pre + "W_down") @ _v_gelu(f(pre + "W_up") @ u + f(pre + "b_up")) + f(pre + "b_down"))
            return out

        if parallel:
            a, m = attn(x), mlp(x)
            x = [x[t] + a[t] + m[t] for t in range(T)]
        else:
            a = attn(x)
            y = [x[t] + a[t] for t in range(T)]
            m = mlp(y)
            x = [y[t] + m[t] for t in range(T)]
    return np.stack(x)


@pytest.mark.parametrize("parallel", [1, 0])
@pytest.mark.parametrize("n_t", [2, 0])
def test_lb1_reduces_to_vanilla(parallel, n_t):
    cfg = tiny_cfg(block_len=1, prefix_len=0, n_block_layers=2, n_token_layers=n_t,
                   parallel_residual=parallel, d_model=16, n_heads=2, d_ff=32, prompt_len=3)
    W = make_weights(cfg)
    P = O.Params(W)
    T = 7
    toks = np.random.default_rng(3).integers(0, cfg.vocab, size=(1, T))
    causal = [[j <= i for j in range(T)] for i in range(T)]
    selfonly = [[j == i for j in range(T)] for i in range(T)]
    stages = [(f"blk.{l}.", causal, list(range(T))) for l in range(2)]
    stages.append(("ln", "blk_lnf_g", "blk_lnf_b"))
    stages += [(f"tok.{l}.", selfonly, [0] * T) for l in range(n_t)]
    stages.append(("ln", "tok_lnf_g", "tok_lnf_b"))
    hid = vanilla_forward(W, np.asarray(W["E_emb"], dtype=np.float64)[toks[0]], stages,
                          cfg.n_heads, cfg.rot, cfg.ln_eps, parallel)
    ref_logits = hid @ np.asarray(W["W_head"], dtype=np.float64).T       # [T, V]; row t predicts x_{t+1}
    for t in range(1, T + 1):
        got = O.next_token_logits_full(P, cfg, toks[:, :t])[0]
        assert np.max(np.abs(got - ref_logits[t - 1])) < TOL
    # cached generation follows the same numbers
    _, lg_c, _ = O.generate_cached(P, cfg, toks[:, :3], 4, forced=toks[:, 3:7])
    for k in range(4):
        assert np.max(np.abs(lg_c[0, k] - ref_logits[2 + k])) < TOL


def test_lb1_identity_prefix_equals_no_prefix():
    cfg0 = tiny_cfg(block_len=1, prefix_len=0, d_model=16, n_heads=2, d_ff=32, prompt_len=3)
    cfg1 = cfg0.with_(prefix_len=1)
    W = make_weights(cfg0)
    W1 = dict(W)
    W1["W_prefix"] = np.eye(16, dtype=np.float32)
    W1["b_prefix"] = np.zeros(16, dtype=np.float32)
    toks = np.random.default_rng(4).integers(0, cfg0.vocab, size=(2, 6))
    a = O.next_token_logits_full(O.Params(W), cfg0, toks)
    b = O.next_token_logits_full(O.Params(W1), cfg1, toks)
    assert np.max(np.abs(a - b)) < TOL


def test_block_model_against_vanilla_pieces():
    """L_B=4, P=2: block decoder == vanilla stack over block embeddings; token decoder ==
    vanilla stack over [prefix, tokens]; glued by concat / projection written out here."""
    cfg = tiny_cfg(block_len=4, prefix_len=2, d_model=16, n_heads=2, d_ff=32, prompt_len=8, vocab=23)
    W = make_weights(cfg)
    P = O.Params(W)
    f = lambda nm: np.asarray(W[nm], dtype=np.float64)
    toks = np.random.default_rng(5).integers(0, cfg.vocab, size=(1, 11))   # 2 full blocks + 3
    nblk = 2
    e = np.stack([np.concatenate([f("E_emb")[toks[0, j * 4 + k]] for k in range(4)]) for j in range(nblk)])
    causal = lambda n: [[j <= i for j in range(n)] for i in range(n)]
    st = [(f"blk.{l}.", causal(nblk), list(range(nblk))) for l in range(cfg.n_block_layers)]
    st.append(("ln", "blk_lnf_g", "blk_lnf_b"))
    ctx = vanilla_forward(W, e, st, cfg.n_heads, cfg.rot, cfg.ln_eps, 1)[-1]
    pre = (f("W_prefix") @ ctx + f("b_prefix")).reshape(2, 16)
    s = np.concatenate([pre, f("E_tok")[toks[0, 8:11]]], axis=0)          # length 2+3 = 5
    st = [(f"tok.{l}.", causal(5), list(range(5))) for l in range(cfg.n_token_layers)]
    st.append(("ln", "tok_lnf_g", "tok_lnf_b"))
    hid = vanilla_forward(W, s, st, cfg.n_heads, cfg.rot, cfg.ln_eps, 1)
    ref = hid @ f("W_head").T
    for r in range(4):          # local position P-1+r predicts token 8+r
        got = O.next_token_logits_full(P, cfg, toks[:, :8 + r])[0]
        assert np.max(np.abs(got - ref[1 + r])) < TOL


# --------------------------------------------------------------------------
# T4  brute-force attention in long double; streaming (split) softmax algebra
# --------------------------------------------------------------------------
def _brute_attention(q, K, V, n_past):
    B, n, H, dh = q.shape
    out = np.zeros(q.shape, dtype=np.longdouble)
    for b in range(B):
        for h in range(H):
            for i in range(n):
                sc = []
                for j in range(n_past + i + 1):
                    acc = np.longdouble(0)
                    for t in range(dh):
                        acc += np.longdouble(q[b, i, h, t]) * np.longdouble(K[b, j, h, t])
                    sc.append(acc / np.sqrt(np.longdouble(dh)))
                m = max(sc)
                w = [np.exp(s - m) for s in sc]
                z = sum(w)
                for j, wj in enumerate(w):
                    for t in range(dh):
                        out[b, i, h, t] += wj / z * np.longdouble(V[b, j, h, t])
    return out.astype(np.float64)


@pytest.mark.parametrize("n_past,n", [(0, 5), (3, 1), (4, 3)])
def test_attention_brute_force(n_past, n):
    rng = np.random.default_rng(6)
    q = rng.standard_normal((2, n, 2, 5)) * 2
    K = rng.standard_normal((2, n_past + n, 2, 5)) * 2
    V = rng.standard_normal((2, n_past + n, 2, 5))
    assert np.max(np.abs(O.attention(q, K, V, n_past) - _brute_attention(q, K, V, n_past))) < 1e-12


@pytest.mark.parametrize("chunks", [1, 2, 3, 7])
def test_split_softmax_combine_matches_attention(chunks):
    """The partial (max, sum, weighted acc) combine used by split-K decoding is exact algebra."""
    rng = np.random.default_rng(7)
    N, dh = 23, 8
    q = rng.standard_normal((1, 1, 1, dh)) * 3
    K = rng.standard_normal((1, N, 1, dh)) * 3
    V = rng.standard_normal((1, N, 1, dh))
    ref = O.attention(q, K, V, N - 1)[0, 0, 0]
    bounds = np.linspace(0, N, chunks + 1).astype(int)
    parts = []
    for a, b in zip(bounds[:-1], bounds[1:]):
        if a == b:
            continue
        s = (K[0, a:b, 0] @ q[0, 0, 0]) / math.sqrt(dh)
        m = s.max()
        w = np.exp(s - m)
        parts.append((m, w.sum(), w @ V[0, a:b, 0]))
    M = max(p[0] for p in parts)
    l = sum(p[1] * math.exp(p[0] - M) for p in parts)
    acc = sum(p[2] * math.exp(p[0] - M) for p in parts)
    assert np.max(np.abs(acc / l - ref)) < 1e-12


# --------------------------------------------------------------------------
# T5  closed forms
# --------------------------------------------------------------------------
def test_zero_query_gives_running_mean():
    rng = np.random.default_rng(8)
    n_past, n = 2, 4
    V = rng.standard_normal((1, n_past + n, 2, 3))
    K = rng.standard_normal((1, n_past + n, 2, 3))
    out = O.attention(np.zeros((1, n, 2, 3)), K, V, n_past)
    for i in range(n):
        assert np.max(np.abs(out[0, i] - V[0, :n_past + i + 1].mean(axis=0))) < 1e-13


def test_layer_closed_form_running_mean_of_v():
    cfg = tiny_cfg(block_len=1, prefix_len=0, d_model=8, n_heads=2, d_ff=16, rotary_dims=0)
    W = make_weights(cfg)
    D = 8
    W["blk.0.W_qkv"][:D] = 0; W["blk.0.b_qkv"][:D] = 0           # q == 0
    W["blk.0.W_o"] = np.eye(D, dtype=np.float32); W["blk.0.b_o"][:] = 0
    W["blk.0.W_down"][:] = 0; W["blk.0.b_down"][:] = 0            # MLP == 0
    P = O.Params(W)
    x = np.random.default_rng(9).standard_normal((1, 5, D))
    out = O.transformer_layer(P, "blk.0.", x, 0, cfg)
    g, b = W["blk.0.ln1_g"].astype(np.float64), W["blk.0.ln1_b"].astype(np.float64)
    u = (x[0] - x[0].mean(-1, keepdims=True)) / np.sqrt(x[0].var(-1, keepdims=True) + cfg.ln_eps) * g + b
    v = u @ W["blk.0.W_qkv"][2 * D:].astype(np.float64).T + W["blk.0.b_qkv"][2 * D:]
    for t in range(5):
        assert np.max(np.abs(out[0, t] - (x[0, t] + v[:t + 1].mean(axis=0)))) < 1e-12


def test_constant_logits_pick_index_zero_and_one_hot_head():
    cfg = tiny_cfg(block_len=2, prefix_len=1, d_model=16, n_heads=2, d_ff=32, prompt_len=4, vocab=16)
    W = make_weights(cfg)
    W["W_head"][:] = 0
    ids, lg, _ = O.generate_cached(O.Params(W), cfg, make_prompts(cfg), 5)
    assert np.all(lg == 0) and np.all(ids == 0)
    # one-hot head: logit v reads hidden unit perm[v]
    perm = np.random.default_rng(10).permutation(16)
    W["W_head"] = np.eye(16, dtype=np.float32)[perm]
    P = O.Params(W)
    toks = make_prompts(cfg)
    c = O.context_embeddings(P, cfg, toks)[:, -1]
    hid = O.token_decoder(P, cfg, O.prefix_tokens(P, cfg, c))[:, -1]
    lg = O.next_token_logits_full(P, cfg, toks)
    assert np.array_equal(lg, hid[:, perm])
    assert np.array_equal(O.greedy(lg), np.array([int(np.where(perm == np.argmax(h))[0][0]) for h in hid]))
    assert O.greedy(np.array([[1.0, 3.0, 3.0, 2.0]]))[0] == 1        # lowest index on ties


# --------------------------------------------------------------------------
# T6  embedder is an exact lookup-and-concatenate (Sec. 2.2)
# --------------------------------------------------------------------------
def test_embedder_exact():
    cfg = tiny_cfg(block_len=4, d_model=32)
    W = make_weights(cfg)
    P = O.Params(W)
    toks = make_prompts(cfg, batch=3, prompt_len=12)
    e = O.embedder(P, cfg, toks)
    assert e.shape == (3, 3, 32)
    de = cfg.d_emb
    assert de == 32 // 4
    for b in range(3):
        for j in range(3):
            for k in range(4):
                assert np.array_equal(e[b, j, k * de:(k + 1) * de], W["E_emb"][toks[b, j * 4 + k]].astype(np.float64))


# --------------------------------------------------------------------------
# T7  operation counts the paper states (Sec. 2.3, 2.4, App. C, attention-map caption)
# --------------------------------------------------------------------------
@pytest.mark.parametrize("lb,p,tp,tg", [(4, 2, 8, 9), (4, 1, 8, 8), (2, 1, 4, 7), (1, 1, 3, 5), (8, 2, 16, 17)])
def test_procedure_counts(lb, p, tp, tg):
    cfg = tiny_cfg(block_len=lb, prefix_len=p, prompt_len=tp, d_model=32, n_heads=2)
    P = build(cfg)
    gen = O.CachedGenerator(P, cfg, 2, (tp + tg) // lb + 1)
    gen.prefill(make_prompts(cfg))
    n_p = tp // lb
    assert gen.token_passes == 0                              # token-decoder prefill is skipped
    assert gen.blk[0].n == n_p                                # one KV entry per block
    for _ in range(tg):
        gen.step()
    extra = -(-tg // lb) - 1
    assert gen.block_passes == n_p + extra
    assert gen.blk[0].n == n_p + extra                        # entries == embedded tokens / L_B
    assert gen.token_passes == tg
    assert gen.local_kv_high_water == min(p + lb - 1, p + tg - 1)
    # cached block entries attended: sum over block steps of (entries incl. the new one)
    assert gen.block_kv_rows_read == sum(n_p + k + 1 for k in range(extra))


def test_kv_ratio_block_vs_vanilla():
    """KV size / L_B, KV access / L_B^2 (Sec. 2.3): closed-form check of the counters."""
    def reads(lb, tp, tg):
        cfg = tiny_cfg(block_len=lb, prefix_len=1, prompt_len=tp, d_model=16, n_heads=2, d_ff=16,
                       n_block_layers=1, n_token_layers=1)
        gen = O.CachedGenerator(build(cfg), cfg, 1, (tp + tg) // lb + 1)
        gen.prefill(make_prompts(cfg, batch=1))
        for _ in range(tg):
            gen.step()
        return gen.block_kv_rows_read, gen.blk[0].n
    r1, n1 = reads(1, 16, 129)
    r4, n4 = reads(4, 16, 129)
    assert abs(n1 / n4 - 4) < 0.2
    assert abs(r1 / r4 - 16) < 1.0        # -> L_B^2 as lengths grow


def test_table3_parameter_counts():
    """Non-embedding sizes printed in the hyper-parameter table (App. E.2)."""
    path = os.path.join(os.path.dirname(__file__), "golden", "table3_sizes.txt")
    rows = [l.split() for l in open(path) if l.strip() and not l.startswith("#")]
    for n_layers, dim, stated_millions in rows:
        n_layers, dim, stated = int(n_layers), int(dim), float(stated_millions)
        cfg = tiny_cfg(d_model=dim, d_ff=4 * dim, n_heads=8, n_block_layers=n_layers, n_token_layers=0,
                       block_len=1, prefix_len=0, vocab=2)
        per_layer = sum(int(np.prod(s)) for nm, s, _ in tensor_table(cfg) if nm.startswith("blk.0."))
        assert per_layer == 12 * dim * dim + 13 * dim
        # the table prints sizes rounded to whole millions (5M stands for 4.74M)
        assert abs(n_layers * per_layer / 1e6 - stated) < max(0.6, 0.01 * stated)


# --------------------------------------------------------------------------
# T8  batch independence
# --------------------------------------------------------------------------
def test_batch_independence():
    cfg = tiny_cfg(block_len=4, prefix_len=2)
    P = build(cfg)
    prompts = make_prompts(cfg, batch=3)
    ids, lg, _ = O.generate_cached(P, cfg, prompts, 6)
    for b in range(3):
        ids1, lg1, _ = O.generate_cached(P, cfg, prompts[b:b + 1], 6)
        assert np.array_equal(ids1[0], ids[b])
        assert np.max(np.abs(lg1[0] - lg[b])) < 1e-12


# --------------------------------------------------------------------------
# T9  rotary: identity at position 0, norm-preserving, relative-position invariance
# --------------------------------------------------------------------------
def test_rotary_properties():
    rng = np.random.default_rng(12)
    x = rng.standard_normal((1, 4, 2, 16))
    y = rng.standard_normal((1, 4, 2, 16))
    assert np.array_equal(O.rotary(x, [0, 0, 0, 0], 8), x)
    r = O.rotary(x, [0, 1, 2, 3], 8)
    assert np.array_equal(r[..., 8:], x[..., 8:])                   # dims beyond rot untouched
    assert np.max(np.abs(np.linalg.norm(r, axis=-1) - np.linalg.norm(x, axis=-1))) < 1e-12
    s0 = np.einsum("bihd,bjhd->bhij", O.rotary(x, [0, 1, 2, 3], 8), O.rotary(y, [0, 1, 2, 3], 8))
    s1 = np.einsum("bihd,bjhd->bhij", O.rotary(x, [5, 6, 7, 8], 8), O.rotary(y, [5, 6, 7, 8], 8))
    assert np.max(np.abs(s0 - s1)) < 1e-12
    # explicit 2-D rotation of the pair (t, t + rot/2) by pos * 10000^(-2t/rot)
    t, pos, rot = 1, 3, 8
    th = pos * 10000.0 ** (-2.0 * t / rot)
    a, b = x[0, 3, 0, t], x[0, 3, 0, t + rot // 2]
    assert abs(r[0, 3, 0, t] - (a * math.cos(th) - b * math.sin(th))) < 1e-14
    assert abs(r[0, 3, 0, t + rot // 2] - (b * math.cos(th) + a * math.sin(th))) < 1e-14


def test_token_decoder_positions_restart_each_block():
    """Token-decoder positions are local: the same (context, block tokens) gives the same
    logits whichever block index it is."""
    cfg = tiny_cfg(block_len=4, prefix_len=1)
    P = build(cfg)
    rng = np.random.default_rng(13)
    toks = rng.integers(0, cfg.vocab, size=(1, 16))
    c = rng.standard_normal((1, cfg.d_model))
    res = []
    for n_prompt in (4, 12):
        g = O.CachedGenerator(P, cfg, 1, 8)
        g.prefill(toks[:, :n_prompt])
        g.c = c.copy()
        res.append(np.stack([g.step(forced_ids=[5])[0] for _ in range(4)]))
    assert np.array_equal(res[0], res[1])


# --------------------------------------------------------------------------
# sanity of LayerNorm / GELU against textbook values
# --------------------------------------------------------------------------
def test_layernorm_gelu_values():
    x = np.array([[1.0, 2.0, 3.0, 6.0]])
    out = O.layer_norm(x, np.ones(4), np.zeros(4), 0.0)
    assert abs(out.mean()) < 1e-15 and abs(out.var() - 1.0) < 1e-12      # biased variance
    assert abs(O.gelu(np.array([0.0]))[0]) == 0.0
    assert abs(O.gelu(np.array([1.0]))[0] - 0.8413447460685429) < 1e-15   # Phi(1)
    assert abs(O.gelu(np.array([-2.0]))[0] + 2 * 0.022750131948179195) < 1e-15


# --------------------------------------------------------------------------
# prompts whose length is not a multiple of L_B (App. "Random length padding";
# footnote of the zero-shot table, Sec. 3)
# --------------------------------------------------------------------------
@pytest.mark.parametrize("lb", [1, 2, 4, 8])
def test_left_pad_count_and_place(lb):
    cfg = tiny_cfg(block_len=lb, prefix_len=1, d_model=32, n_heads=2).with_(pad_id=7)
    for T in range(1, 2 * lb + 2):
        toks = 100 + np.arange(2 * T).reshape(2, T)
        out = O.left_pad(cfg, toks)
        assert out.shape[1] % lb == 0 and 0 <= out.shape[1] - T < lb      # fewest pads that fill the block
        assert np.array_equal(out[:, out.shape[1] - T:], toks)            # prompt keeps its order, at the end
        assert np.all(out[:, :out.shape[1] - T] == 7)                     # pads in front
    assert O.left_pad(cfg, np.array([[3]])).shape[1] == lb                # one token: L_B - 1 pads (footnote)


@pytest.mark.parametrize("lb,T", [(4, 1), (4, 6), (4, 7), (2, 5), (8, 3)])
def test_ragged_prompt_equals_hand_padded_prompt(lb, T):
    """Full and cached generation from T tokens == generation from the block-aligned prompt
    written out by hand, and differs from padding on the right."""
    cfg = tiny_cfg(block_len=lb, prefix_len=1, d_model=32, n_heads=2, prompt_len=T).with_(pad_id=5)
    P = build(cfg)
    toks = make_prompts(cfg, batch=2)
    k = -(-T // lb) * lb - T
    by_hand = np.array([[5] * k + [int(t) for t in row] for row in toks])
    ids_a, lg_a = O.generate_full(P, cfg, toks, lb + 2)
    ids_b, lg_b = O.generate_full(P, cfg, by_hand, lb + 2)
    assert np.array_equal(lg_a, lg_b) and np.array_equal(ids_a, ids_b)
    ids_c, lg_c, gen = O.generate_cached(P, cfg, toks, lb + 2)
    assert np.array_equal(ids_c, ids_a) and np.abs(lg_c - lg_a).max() < 1e-11
    assert gen.blk[0].n == (T + k) // lb + 1
    right = np.array([[int(t) for t in row] + [5] * k for row in toks])
    assert np.abs(O.generate_full(P, cfg, right, 1)[1] - lg_a[:, :1]).max() > 1e-6


def test_pad_tokens_enter_the_first_block_embedding():
    """Unlike masked pads of a vanilla transformer, the pad id's embedding is part of the first
    block's input: the row is the concatenation of table rows, pads included."""
    cfg = tiny_cfg(block_len=4, prefix_len=1, d_model=32, n_heads=2, prompt_len=6).with_(pad_id=9)
    W = make_weights(cfg)
    P = O.Params(W)
    toks = make_prompts(cfg, batch=1)
    e = O.embedder(P, cfg, O.left_pad(cfg, toks))
    E = W["E_emb"].astype(np.float64)
    want = np.concatenate([E[9], E[9], E[int(toks[0, 0])], E[int(toks[0, 1])]])
    assert np.array_equal(e[0, 0], want)
    other = O.generate_full(P, cfg.with_(pad_id=10), toks, 1)[1]
    assert np.abs(other - O.generate_full(P, cfg, toks, 1)[1]).max() > 1e-6


def test_ragged_batch_is_each_sequence_alone():
    """A batch of prompts of different lengths == every sequence run by the no-cache definition on
    its own hand-padded prompt; with equal lengths it is the ordinary batch."""
    cfg = tiny_cfg(block_len=4, prefix_len=2, d_model=32, n_heads=2, prompt_len=11).with_(pad_id=2)
    P = build(cfg)
    full = make_prompts(cfg, batch=4)
    lens = [11, 1, 8, 6]
    prompts = [full[b, :n] for b, n in enumerate(lens)]
    ids, lgs = O.generate_ragged(P, cfg, prompts, 6)
    for b, n in enumerate(lens):
        k = (-n) % 4
        by_hand = np.array([[2] * k + [int(t) for t in prompts[b]]])
        i1, l1 = O.generate_full(P, cfg, by_hand, 6)
        assert np.array_equal(ids[b], i1[0]) and np.abs(lgs[b] - l1[0]).max() < 1e-11
    same = [full[b, :8] for b in range(4)]
    ids2, lgs2 = O.generate_ragged(P, cfg, same, 5)
    ids3, lgs3, _ = O.generate_cached(P, cfg, full[:, :8], 5)
    assert np.array_equal(ids2, ids3) and np.abs(lgs2 - lgs3).max() < 1e-11


def test_eos_rule():
    """eos_id = -1 changes nothing; with an eos id the ids equal the free run up to and including
    each sequence's first eos and are eos afterwards; other sequences are untouched."""
    cfg = tiny_cfg(block_len=4, prefix_len=1, d_model=32, n_heads=2, prompt_len=8, vocab=13)
    P = build(cfg)
    toks = make_prompts(cfg, batch=3)
    free, lg_free, _ = O.generate_cached(P, cfg, toks, 14)
    eos = int(free[0, 5])                                   # sequence 0 emits it at step <= 5
    ids, lgs, gen = O.generate_cached(P, cfg.with_(eos_id=eos), toks, 14)
    hits = 0
    for b in range(3):
        where = np.nonzero(free[b] == eos)[0]
        if len(where) == 0:
            assert np.array_equal(ids[b], free[b]) and not gen.finished[b]
            continue
        k = where[0]
        hits += 1
        assert np.array_equal(ids[b, :k + 1], free[b, :k + 1])
        assert np.all(ids[b, k:] == eos) and gen.finished[b]
        assert np.array_equal(lgs[b, :k + 1], lg_free[b, :k + 1])
    assert hits >= 1 and np.all(ids[0, 5:] == eos)


# --------------------------------------------------------------------------
# teacher-forced scoring (Sec. 2.1: all blocks in parallel)
# --------------------------------------------------------------------------
def test_score_nll_against_stepwise_definition_and_closed_forms():
    cfg = tiny_cfg(block_len=4, prefix_len=2, d_model=32, n_heads=2, prompt_len=12, vocab=19)
    W = make_weights(cfg)
    P = O.Params(W)
    toks = make_prompts(cfg, batch=2)
    nll = O.score_nll(P, cfg, toks)
    assert nll.shape == (2, 12) and np.all(nll[:, :4] == 0.0) and np.all(nll[:, 4:] > 0.0)
    # position by position from the one-step definition, softmax written out with math.log / math.exp
    for t in (4, 5, 7, 8, 11):
        lg = O.next_token_logits_full(P, cfg, toks[:, :t])
        for b in range(2):
            z = [float(v) for v in lg[b]]
            den = sum(math.exp(v - max(z)) for v in z)
            want = -(z[int(toks[b, t])] - max(z) - math.log(den))
            assert abs(nll[b, t] - want) < 1e-12
    # a head of zeros gives the uniform distribution: nll = log V everywhere
    W0 = dict(W)
    W0["W_head"] = np.zeros_like(W["W_head"])
    assert np.allclose(O.score_nll(O.Params(W0), cfg, toks)[:, 4:], math.log(19), atol=1e-12)
    # probabilities of one position sum to one when the target runs over the vocabulary
    base = toks[:1].copy()
    tot = 0.0
    for v in range(19):
        base[0, 6] = v
        tot += math.exp(-O.score_nll(P, cfg, base)[0, 6])
    assert abs(tot - 1.0) < 1e-12


def test_score_nll_of_a_length_that_is_not_whole_blocks():
    """Scoring T tokens == scoring the hand-padded sequence and dropping the pads' entries."""
    cfg = tiny_cfg(block_len=4, prefix_len=1, d_model=32, n_heads=2, prompt_len=10, vocab=19).with_(pad_id=6)
    P = build(cfg)
    toks = make_prompts(cfg, batch=2)
    by_hand = np.array([[6, 6] + [int(t) for t in row] for row in toks])
    a = O.score_nll(P, cfg, toks)
    b = O.score_nll(P, cfg, by_hand)
    assert a.shape == (2, 10) and np.array_equal(a, b[:, 2:])
    assert np.all(a[:, :2] == 0.0) and np.all(a[:, 2:] > 0.0)      # first block = 2 pads + 2 tokens: those 2 are not scored


# --------------------------------------------------------------------------
# bf16 storage: the path by which bf16-mode weights reach the oracle's float64 arithmetic
# (weights are drawn in float32, rounded to the nearest bf16 with ties to even, stored as
# bit patterns, and widened exactly).  The format is fixed: 1 sign, 8 exponent, 7 mantissa bits,
# the upper half of an IEEE float32.  Values below are worked out by hand from that definition.
# --------------------------------------------------------------------------
def test_bf16_bit_patterns_widen_to_hand_computed_values():
    from synth import bf16_bits_to_f32
    pats = np.array([0x3F80, 0xC000, 0x3DCD, 0x0001, 0x0000, 0x8000, 0x7F7F, 0x0080, 0x4049], dtype=np.uint16)
    want = np.array([
        1.0,                                   # exponent 127, mantissa 0
        -2.0,                                  # sign, exponent 128
        (1.0 + 77.0 / 128.0) * 2.0 ** -4,      # 0x3DCD: exponent 123, mantissa 0x4D = 77 -> 0.10009765625
        2.0 ** -133,                           # smallest subnormal: 2^-126 * 1/128
        0.0, -0.0,
        (2.0 - 2.0 ** -7) * 2.0 ** 127,        # largest finite
        2.0 ** -126,                           # smallest normal
        (1.0 + 73.0 / 128.0) * 2.0,            # 0x4049 = 3.140625
    ])
    assert want[2] == 0.10009765625 and want[8] == 3.140625
    got = bf16_bits_to_f32(pats)
    assert got.dtype == np.float32 and np.array_equal(got.astype(np.float64), want)
    assert np.signbit(got[5]) and not np.signbit(got[4])
    # the oracle's own widening (Params) gives the same float64 values, for any array shape
    P = O.Params({"w": pats.reshape(3, 3)})
    w = P("w")
    assert w.dtype == np.float64 and np.array_equal(w.ravel(), want) and np.signbit(w.ravel()[5])
    # float32 arrays pass through Params unchanged in value
    f = np.array([0.1, -3.5, 1e-30], dtype=np.float32)
    assert np.array_equal(O.Params({"f": f})("f"), f.astype(np.float64))


def test_f32_to_bf16_rounds_to_nearest_even():
    from synth import bf16_bits_to_f32, f32_to_bf16_bits
    def f32(bits):
        return np.array([bits], dtype=np.uint32).view(np.float32)
    cases = [
        (f32(0x3F808000), 0x3F80),     # 1 + 2^-8: exactly between 0x3F80 and 0x3F81 -> the even one
        (f32(0x3F818000), 0x3F82),     # 1 + 3*2^-8: between 0x3F81 and 0x3F82 -> even
        (f32(0x3F808001), 0x3F81),     # just above the tie -> up
        (f32(0x3F807FFF), 0x3F80),     # just below -> down
        (f32(0x3FFFFFFF), 0x4000),     # just under 2: the carry runs into the exponent
        (f32(0x7F7FFFFF), 0x7F80),     # largest float32 rounds to +inf, as IEEE rounding does
        (f32(0xBF808000), 0xBF80),     # ties are symmetric in sign
        (f32(0x00000000), 0x0000), (f32(0x80000000), 0x8000),
        (np.array([0.1], dtype=np.float32), 0x3DCD),      # 0.1f = 0x3DCCCCCD -> 0x3DCD
    ]
    for x, want in cases:
        assert int(f32_to_bf16_bits(x)[0]) == want, (hex(int(x.view(np.uint32)[0])), hex(want))
    # every non-NaN bf16 value survives widening and rounding back unchanged (65 280 patterns)
    allp = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    is_nan = ((allp & 0x7F80) == 0x7F80) & ((allp & 0x007F) != 0)
    p = allp[~is_nan]
    assert p.size == 65536 - 2 * 127
    assert np.array_equal(f32_to_bf16_bits(bf16_bits_to_f32(p)), p)
    # rounding error is at most half a unit in the last of 8 significant bits
    rng = np.random.default_rng(3)
    x = (rng.standard_normal(20000) * 0.02).astype(np.float32)
    back = bf16_bits_to_f32(f32_to_bf16_bits(x)).astype(np.float64)
    assert np.all(np.abs(back - x) <= np.abs(x.astype(np.float64)) * 2.0 ** -8)
    # and it is the NEAREST bf16: neither neighbour is closer
    bits = f32_to_bf16_bits(x).astype(np.int64)
    for d in (-1, 1):
        nb = bf16_bits_to_f32((bits + d).astype(np.uint16)).astype(np.float64)
        assert np.all(np.abs(back - x) <= np.abs(nb - x))


@pytest.mark.parametrize("lb,p", [(4, 2), (1, 0)])
def test_cached_equals_full_with_bf16_weights(lb, p):
    """The same T1 check through the bf16 storage path, and against float32 weights holding the
    widened values: the oracle sees bf16-mode weights as exactly those numbers."""
    from synth import bf16_bits_to_f32
    cfg = tiny_cfg(dtype="bf16", block_len=lb, prefix_len=p, prompt_len=2 * lb, d_model=32, n_heads=2)
    W = make_weights(cfg)
    assert W["W_head"].dtype == np.uint16 and W["blk.0.W_qkv"].dtype == np.uint16 and W["blk.0.b_qkv"].dtype == np.float32
    prompts = make_prompts(cfg, batch=3)
    n_new = 2 * lb + 3
    ids_f, lg_f = O.generate_full(O.Params(W), cfg, prompts, n_new)
    ids_c, lg_c, _ = O.generate_cached(O.Params(W, keep=False), cfg, prompts, n_new)
    assert np.array_equal(ids_f, ids_c) and np.max(np.abs(lg_f - lg_c)) < TOL
    W32 = {k: (bf16_bits_to_f32(v) if v.dtype == np.uint16 else v) for k, v in W.items()}
    ids_w, lg_w = O.generate_full(O.Params(W32), cfg.with_(dtype="fp32"), prompts, n_new)
    assert np.array_equal(ids_f, ids_w) and np.array_equal(lg_f, lg_w)
    # the rounding is really there: the float32 draw of the same seed gives other logits
    Wf = make_weights(cfg.with_(dtype="fp32"))
    assert np.array_equal(bf16_bits_to_f32(W["W_head"]), bf16_bits_to_f32(__import__("synth").f32_to_bf16_bits(Wf["W_head"])))
    _, lg_u = O.generate_full(O.Params(Wf), cfg.with_(dtype="fp32"), prompts, 1)
    assert np.max(np.abs(lg_u - lg_f[:, :1])) > 1e-6


# --------------------------------------------------------------------------
# Summation token decoder (App. D.2 "Summation"): the context embedding, projected to L_B vectors,
# is added to the token decoder's inputs position by position.
# --------------------------------------------------------------------------
def _sum_cfg(**kw):
    base = dict(block_len=4, prefix_len=1, token_mix="sum", d_model=32, n_heads=2, prompt_len=8)
    base.update(kw)
    return tiny_cfg(**base)


@pytest.mark.parametrize("lb", [1, 2, 4])
@pytest.mark.parametrize("parallel", [1, 0])
def test_summation_cached_equals_full(lb, parallel):
    cfg = _sum_cfg(block_len=lb, prompt_len=2 * lb, parallel_residual=parallel)
    W = make_weights(cfg)
    assert W["W_prefix"].shape == (lb * cfg.d_model, cfg.d_model) and W["b_prefix"].shape == (lb * cfg.d_model,)
    P = O.Params(W)
    prompts = make_prompts(cfg, batch=3)
    n_new = 2 * lb + 3
    ids_f, lg_f = O.generate_full(P, cfg, prompts, n_new)
    ids_c, lg_c, gen = O.generate_cached(P, cfg, prompts, n_new)
    assert np.array_equal(ids_f, ids_c) and np.max(np.abs(lg_f - lg_c)) < TOL
    assert gen.local_kv_high_water == lb                      # positions 0 .. L_B - 1: no prefix row besides position 0


def test_summation_is_the_one_prefix_model_plus_added_vectors():
    """With summands 1 .. L_B-1 zeroed the variant IS the prefix model with one prefix token whose
    projection is summand 0; a non-zero summand k changes the logits of positions >= k only (the
    token decoder is causal inside the block)."""
    cfg = _sum_cfg()
    D, L = cfg.d_model, cfg.block_len
    W = make_weights(cfg)
    rng = np.random.default_rng(4)
    toks = rng.integers(0, cfg.vocab, size=(2, 12))
    Wz = dict(W)
    Wz["W_prefix"] = W["W_prefix"].copy(); Wz["b_prefix"] = W["b_prefix"].copy()
    Wz["W_prefix"][D:] = 0; Wz["b_prefix"][D:] = 0
    pcfg = cfg.with_(token_mix="prefix")
    Wp = dict(W)
    Wp["W_prefix"] = W["W_prefix"][:D].copy(); Wp["b_prefix"] = W["b_prefix"][:D].copy()
    a = O.teacher_forced_logits(O.Params(Wz), cfg, toks, [1, 2])
    b = O.teacher_forced_logits(O.Params(Wp), pcfg, toks, [1, 2])
    for i in (1, 2):
        assert np.max(np.abs(a[i] - b[i])) < TOL
    # the full variant differs from it, and summand k alone moves positions >= k
    full = O.teacher_forced_logits(O.Params(W), cfg, toks, [1, 2])
    assert np.max(np.abs(full[1] - a[1])) > 1e-6
    for k in range(1, L):
        Wk = dict(Wz)
        Wk["W_prefix"] = Wz["W_prefix"].copy(); Wk["b_prefix"] = Wz["b_prefix"].copy()
        Wk["W_prefix"][k * D:(k + 1) * D] = W["W_prefix"][k * D:(k + 1) * D]
        Wk["b_prefix"][k * D:(k + 1) * D] = W["b_prefix"][k * D:(k + 1) * D]
        ck = O.teacher_forced_logits(O.Params(Wk), cfg, toks, [2])[2]
        assert np.max(np.abs(ck[:, :k] - a[2][:, :k])) == 0.0
        assert np.min(np.max(np.abs(ck[:, k:] - a[2][:, k:]), axis=-1)) > 1e-9


def test_summation_inputs_written_out():
    """The token decoder's input rows of one block, element by element."""
    cfg = _sum_cfg()
    D, L = cfg.d_model, cfg.block_len
    W = make_weights(cfg)
    P = O.Params(W)
    rng = np.random.default_rng(5)
    c = rng.standard_normal((2, D))
    blk = rng.integers(0, cfg.vocab, size=(2, 3))
    s = O.local_inputs(P, cfg, c, blk)
    assert s.shape == (2, 4, D)
    for b in range(2):
        for k in range(4):
            want = np.array([sum(W["W_prefix"][k * D + d, j].astype(np.float64) * c[b, j] for j in range(D)) + W["b_prefix"][k * D + d]
                             for d in range(D)])
            if k >= 1:
                want = want + W["E_tok"][blk[b, k - 1]]
            assert np.max(np.abs(s[b, k] - want)) < 1e-12
    # locality: the logits of a block depend on earlier blocks only through the context embedding
    lg1 = O.block_logits(P, cfg, c, blk)
    lg2 = O.block_logits(P, cfg, c, blk.copy())
    assert np.array_equal(lg1, lg2)


def test_summation_at_block_length_one_is_the_one_prefix_model():
    cfg = _sum_cfg(block_len=1, prompt_len=3)
    W = make_weights(cfg)
    prompts = make_prompts(cfg, batch=2)
    _, a = O.generate_full(O.Params(W), cfg, prompts, 5)
    _, b = O.generate_full(O.Params(W), cfg.with_(token_mix="prefix"), prompts, 5)
    assert np.array_equal(a, b)
